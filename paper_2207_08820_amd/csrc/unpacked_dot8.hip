// Comparison variant: the same integer GEMM on UNPACKED 4-bit values with the VALU's 8-way dot product
// (v_dot8_i32_i4: eight signed 4-bit products summed into an int32 per lane and instruction), no bitplanes.
//
// Section V of arXiv 2207.08820 computes sum_k a_k * w_k bit-serially, abits * wbits / 16 VALU lane-ops per
// multiply-add.  The dot instruction costs 1 / 8 whatever the bit widths (up to 4), so on paper it ties with the
// bit-serial form at abits * wbits = 2 and wins above; this kernel is the measurement of that, next to the
// matrix-instruction variant (unpacked_mfma.hip).  Not the product path.
//
// Operands: one signed nibble per element, element k in bits 4 (k % 8) .. 4 (k % 8) + 3 of word k / 8, rows
// K-contiguous (dlrt_pack_nibbles makes them from int8).  NT GEMM: C[m][n] = sum_k A[m][k] * W[n][k], int32.
// 256 threads = 16 x 16 lanes, block tile 128 x 128, lane tile 8 x 8 (rows ty + 16 r, columns tx + 16 s: 64
// accumulators, so that an LDS read feeds 32 dot instructions), K chunks of 256 elements (128 bytes per row)
// staged through LDS, double buffered, laid out [16-byte unit][row] so that neighbouring lanes read and write
// neighbouring 16-byte units.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlrt.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;
constexpr int BM = 128, BN = 128;
constexpr int kUnits = 8;                 // 16-byte units (32 elements) per row and chunk
constexpr int kTile = kUnits * BM;        // units per operand and buffer

__device__ __forceinline__ int dot8(uint32_t a, uint32_t b, int c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_sdot8((int)a, (int)b, c, false);
#else
    (void)a; (void)b;
    return c;  // host pass of the single-source compile: never executed
#endif
}

// K8: words (8 elements each) per row, a multiple of 4
__global__ __launch_bounds__(kThreads) void gemm_i4_dot8_kernel(const uint32_t *A, const uint32_t *W, int32_t *C, int M, int N,
                                                                int K8)
{
    __shared__ uint4 lds[2][2][kTile];  // [buffer][A | W][unit * 128 + row]

    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int tilesN = (N + BN - 1) / BN;
    const int tileM = blockIdx.x / tilesN, tileN = blockIdx.x - tileM * tilesN;
    const int m0 = tileM * BM, n0 = tileN * BN;
    const int units = K8 >> 2;  // 16-byte units per row

    // staging: 1024 units per operand and chunk, 4 per thread.  8 consecutive threads take 8 consecutive rows of one
    // unit (one conflict-free 128-byte LDS write), the next thread bits walk along K (a row's 128 bytes)
    const uint4 *srcA[4], *srcW[4];
    int dst[4], unit_of[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int s = tid + kThreads * t;
        const int row = (s >> 6) * 8 + (s & 7), unit = (s >> 3) & 7;
        dst[t] = unit * BM + row;
        unit_of[t] = unit;
        srcA[t] = reinterpret_cast<const uint4 *>(A) + (size_t)min(m0 + row, M - 1) * units;
        srcW[t] = reinterpret_cast<const uint4 *>(W) + (size_t)min(n0 + row, N - 1) * units;
    }
    uint4 stA[4], stW[4];
    auto fetch = [&](int u0) {  // first unit of the chunk
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int u = u0 + unit_of[t];
            const bool ok = u < units;  // a unit beyond the reduction reads the row's first unit and is discarded
            const uint4 a = srcA[t][ok ? u : 0], w = srcW[t][ok ? u : 0];
            stA[t] = ok ? a : make_uint4(0u, 0u, 0u, 0u);
            stW[t] = ok ? w : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            lds[buf][0][dst[t]] = stA[t];
            lds[buf][1][dst[t]] = stW[t];
        }
    };

    int acc[8][8];
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int s = 0; s < 8; ++s) acc[r][s] = 0;

    const int nchunks = (units + kUnits - 1) / kUnits;
    fetch(0);
    commit(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < nchunks) fetch((c + 1) * kUnits);
        const uint4 *la = lds[buf][0] + ty, *lw = lds[buf][1] + tx;
#pragma unroll 1
        for (int u = 0; u < kUnits; ++u) {  // not unrolled: one unit's operands (64 registers) live at a time
            uint4 a[8], w[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) a[r] = la[u * BM + 16 * r];
#pragma unroll
            for (int s = 0; s < 8; ++s) w[s] = lw[u * BN + 16 * s];
#pragma unroll
            for (int r = 0; r < 8; ++r)
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    int t = acc[r][s];
                    t = dot8(a[r].x, w[s].x, t);
                    t = dot8(a[r].y, w[s].y, t);
                    t = dot8(a[r].z, w[s].z, t);
                    t = dot8(a[r].w, w[s].w, t);
                    acc[r][s] = t;
                }
        }
        if (c + 1 < nchunks) commit(buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int m = m0 + ty + 16 * r;
        if (m >= M) continue;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int n = n0 + tx + 16 * s;
            if (n < N) C[(size_t)m * N + n] = acc[r][s];
        }
    }
}

// int8 values in [-8, 7] -> nibbles: one lane per output word (8 elements, one 8-byte load)
__global__ __launch_bounds__(kThreads) void pack_nibbles_kernel(const int8_t *src, uint32_t *dst, int64_t words)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= words) return;
    const uint2 v = reinterpret_cast<const uint2 *>(src)[i];
    uint32_t out = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        out |= ((v.x >> (8 * e)) & 0xfu) << (4 * e);
        out |= ((v.y >> (8 * e)) & 0xfu) << (4 * e + 16);
    }
    dst[i] = out;
}

}  // namespace

namespace dlrt {

dlrt_status launch_unpacked_gemm_i4(const uint32_t *A, const uint32_t *W, int32_t *C, int M, int N, int K, hipStream_t stream)
{
    const int64_t tiles = (int64_t)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    if (tiles > 0x7fffffffLL) return DLRT_ERR_SHAPE;
    return enqueue(gemm_i4_dot8_kernel, dim3((unsigned)tiles), dim3(kThreads), 0, stream, A, W, C, M, N, K / 8);
}

dlrt_status launch_pack_nibbles(const int8_t *src, int64_t rows, int64_t K, uint32_t *dst, hipStream_t stream)
{
    const int64_t words = rows * (K / 8), blocks = (words + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return DLRT_ERR_SHAPE;
    return enqueue(pack_nibbles_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, src, dst, words);
}

}  // namespace dlrt
