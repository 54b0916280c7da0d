// Per-output-channel dequantize / requantize epilogue for gfx950.
//
// Section IV of arXiv 2207.08820: t_hat = t_bar * s turns the integer accumulator back into a
// real value; the same section's quantizer round(clip(.)) then produces the next layer's
// low-bit activations.  One fused multiply-add on the exactly converted integer, so the fp32
// result is the correctly rounded value of acc * scale + bias.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlrt.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float dequant(int acc, float s, float b) { return __fmaf_rn((float)acc, s, b); }

__device__ __forceinline__ uint32_t requant(float y, float qmax)
{
    return (uint32_t)fminf(fmaxf(rintf(y), 0.0f), qmax);
}

// C % 4 == 0 and 16-byte aligned buffers: four channels per lane, 16-byte accesses.
__global__ __launch_bounds__(kThreads) void epilogue_vec4(const int4 *acc, const float4 *scale, const float4 *bias,
                                                          int64_t n4, int C4, float4 *out_f32, uint32_t *out_q,
                                                          float qmax)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kThreads) {
        const int c = (int)(i % C4);
        const int4 a = acc[i];
        const float4 s = scale[c];
        const float4 b = bias ? bias[c] : make_float4(0.f, 0.f, 0.f, 0.f);
        const float4 y = make_float4(dequant(a.x, s.x, b.x), dequant(a.y, s.y, b.y), dequant(a.z, s.z, b.z),
                                     dequant(a.w, s.w, b.w));
        if (out_f32) out_f32[i] = y;
        if (out_q)
            out_q[i] = requant(y.x, qmax) | requant(y.y, qmax) << 8 | requant(y.z, qmax) << 16 | requant(y.w, qmax) << 24;
    }
}

__global__ __launch_bounds__(kThreads) void epilogue_scalar(const int32_t *acc, const float *scale, const float *bias,
                                                            int64_t n, int C, float *out_f32, uint8_t *out_q,
                                                            float qmax)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) {
        const int c = (int)(i % C);
        const float y = dequant(acc[i], scale[c], bias ? bias[c] : 0.0f);
        if (out_f32) out_f32[i] = y;
        if (out_q) out_q[i] = (uint8_t)requant(y, qmax);
    }
}

bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

}  // namespace

namespace dlrt {

dlrt_status launch_epilogue(const int32_t *acc, const float *scale, const float *bias, int64_t rows, int C,
                            float *out_f32, uint8_t *out_q, int qbits, hipStream_t stream)
{
    const int64_t n = rows * C;
    const float qmax = (float)((1 << qbits) - 1);
    const bool vec = C % 4 == 0 && aligned16(acc) && aligned16(scale) && (!bias || aligned16(bias)) &&
                     (!out_f32 || aligned16(out_f32)) && (!out_q || reinterpret_cast<uintptr_t>(out_q) % 4 == 0);
    const int64_t work = vec ? n / 4 : n;
    int64_t blocks = (work + kThreads - 1) / kThreads;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks < 1) blocks = 1;
    if (vec)
        return enqueue(epilogue_vec4, dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                       reinterpret_cast<const int4 *>(acc), reinterpret_cast<const float4 *>(scale),
                       reinterpret_cast<const float4 *>(bias), work, C / 4, reinterpret_cast<float4 *>(out_f32),
                       reinterpret_cast<uint32_t *>(out_q), qmax);
    return enqueue(epilogue_scalar, dim3((unsigned)blocks), dim3(kThreads), 0, stream, acc, scale, bias, n, C, out_f32,
                   out_q, qmax);
}

}  // namespace dlrt
