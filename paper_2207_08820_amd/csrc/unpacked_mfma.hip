// Comparison variant: the same integer GEMM on the UNPACKED low-bit values with int8 matrix
// instructions (v_mfma_i32_16x16x64_i8), no bitplanes.
//
// Section V of arXiv 2207.08820 computes sum_k a_k * w_k bit-serially because Arm CPUs have no
// low-bit multiply; the bit-serial form costs a*w/16 VALU lane-ops per multiply-add.  On gfx950 the
// matrix cores multiply int8 directly, and 1-4 bit values are valid int8, so this kernel is the
// yardstick that shows at which bit widths the bit-serial path still pays on this chip.  It is kept
// because the measurement says it wins (see the profile summary), not as the product path.
//
// NT GEMM, both operands K-contiguous int8: C[m][n] = sum_k A[m][k] * W[n][k], int32.
// 256 threads = 2 x 2 waves, block tile 128 x 128, wave tile 64 x 64 = 4 x 4 MFMA tiles, K chunks
// of 128 staged through LDS (double buffered, 16-byte units XOR-swizzled by row so that both the
// 128-byte row writes and the 16-lane fragment reads are conflict-free).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlrt.h"
#include "launch.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BM = 128, BN = 128, BK = 128;
constexpr int kUnitsPerRow = BK / 16;            // 8 sixteen-byte units per staged row
constexpr int kTile = BM * kUnitsPerRow;         // units per operand per buffer

__device__ __forceinline__ v4i mfma_i8(v4i a, v4i b, v4i c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
#else
    (void)a; (void)b;
    return c;  // host pass of the single-source compile: never executed
#endif
}

__global__ __launch_bounds__(kThreads) void gemm_i8_mfma_kernel(const int8_t *A, const int8_t *W, int32_t *C, int M, int N,
                                                                int K)
{
    __shared__ uint4 lds[2][2][kTile];  // [buffer][A | W][row * 8 + (unit ^ (row & 7))]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tilesN = (N + BN - 1) / BN;
    const int tileM = blockIdx.x / tilesN, tileN = blockIdx.x - tileM * tilesN;
    const int m0 = tileM * BM, n0 = tileN * BN;

    // staging: 1024 units per operand per chunk, 4 per thread; 8 consecutive threads move one row's 128 bytes
    const int8_t *srcA[4], *srcW[4];
    int dst[4], unitk[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int idx = tid + kThreads * t;
        const int row = idx >> 3, unit = idx & 7;
        dst[t] = row * kUnitsPerRow + (unit ^ (row & 7));
        unitk[t] = unit * 16;
        srcA[t] = A + (size_t)min(m0 + row, M - 1) * K + unit * 16;
        srcW[t] = W + (size_t)min(n0 + row, N - 1) * K + unit * 16;
    }
    uint4 stA[4], stW[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bool ok = k0 + unitk[t] < K;  // K is a multiple of 16: a unit is inside or outside as a whole
            // a unit outside the reduction reads the first 16 bytes of its own row instead (always inside the
            // buffer, since K >= 16) and is discarded; srcA / srcW already point at this thread's unit
            const int kk = ok ? k0 : -unitk[t];
            const uint4 a = *reinterpret_cast<const uint4 *>(srcA[t] + kk);
            const uint4 w = *reinterpret_cast<const uint4 *>(srcW[t] + kk);
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

    v4i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    // fragment addressing: lane (i = lane % 16, g = lane / 16) supplies 16 consecutive k of row i
    const int fi = lane & 15, fg = lane >> 4;
    const int nchunks = (K + BK - 1) / BK;
    fetch(0);
    commit(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < nchunks) fetch((c + 1) * BK);
#pragma unroll
        for (int s = 0; s < BK / 64; ++s) {
            v4i a[4], b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int ra = wm * 64 + t * 16 + fi, rb = wn * 64 + t * 16 + fi;
                const int unit = (4 * s + fg) ^ (fi & 7);  // rows are multiples of 16 plus fi: row & 7 == fi & 7
                const uint4 ua = lds[buf][0][ra * kUnitsPerRow + unit], ub = lds[buf][1][rb * kUnitsPerRow + unit];
                a[t] = v4i{(int)ua.x, (int)ua.y, (int)ua.z, (int)ua.w};
                b[t] = v4i{(int)ub.x, (int)ub.y, (int)ub.z, (int)ub.w};
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = mfma_i8(a[i], b[j], acc[i][j]);
        }
        if (c + 1 < nchunks) commit(buf ^ 1);
        __syncthreads();
    }

    // D[i][j] of a 16 x 16 tile: lane holds column j = lane % 16, rows 4 * (lane / 16) + r
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = m0 + wm * 64 + i * 16 + 4 * fg + r;
            if (m >= M) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = n0 + wn * 64 + j * 16 + fi;
                if (n < N) C[(size_t)m * N + n] = acc[i][j][r];
            }
        }
}

}  // namespace

namespace dlrt {

dlrt_status launch_unpacked_gemm_i8(const int8_t *A, const int8_t *W, int32_t *C, int M, int N, int K, hipStream_t stream)
{
    const int64_t tiles = (int64_t)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    if (tiles > 0x7fffffffLL) return DLRT_ERR_SHAPE;
    return enqueue(gemm_i8_mfma_kernel, dim3((unsigned)tiles), dim3(kThreads), 0, stream, A, W, C, M, N, K);
}

}  // namespace dlrt
