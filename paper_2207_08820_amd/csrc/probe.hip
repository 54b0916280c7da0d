// Measurement probes for bench.py: NOT part of the product library (built into libdlrt_probe.so, which
// nothing but the benchmark loads).  They pin the denominators the bit-serial kernels are judged against
// on the chip that runs the benchmark:
//   * dlrt_probe_valu   - a register-only loop of the contraction's own instruction pair, v_and_b32 +
//                         accumulating v_bcnt_u32_b32 (Section V of arXiv 2207.08820 costs exactly one such
//                         pair per plane pair and 32 reduction elements): the lane-op rate the VALUs sustain
//                         at a given number of waves per SIMD, and, from the shader-clock and constant-rate
//                         counters read at both ends of the loop, the clock the chip really ran at;
//   * dlrt_probe_gemm_clocks - the library's own block kernel (contract.hip, built a second time into this
//                         library with DLRT_CLOCK_PROBE) on a packed GEMM, every block leaving its lifetime on
//                         both counters: the clock during the kernel the roofline fraction is quoted for (after
//                         an idle spell the chip takes tens of milliseconds of load to reach its steady clock, so
//                         a fraction of the nominal peak means little without it);
//   * dlrt_probe_copy   - a plain device copy: the HBM bandwidth a simple kernel reaches;
//   * dlrt_probe_empty  - an empty kernel: the floor of a dependent launch.
// Like the library, every call only enqueues on the caller's stream; bench.py does the timing.
//
//   int  dlrt_probe_valu(int blocks, int iters, uint64_t *clocks /* device, 2 per block */, uint32_t *sink /* device, 256 per block */, void *stream);
//   int  dlrt_probe_gemm_clocks(const uint32_t *A, const uint32_t *W, int32_t *C, int M, int N, int K, int abits, int wbits,
//                               uint64_t *clocks /* device, 2 per tile of (64 or, for 3 and 4 bits, 32) rows x columns */, void *stream);
//                               unsigned activations, two's-complement weights, M, N multiples of 64, K of 128, 16-byte aligned
//   int  dlrt_probe_copy(const void *src, void *dst, size_t bytes /* multiple of 16 */, void *stream);
//   int  dlrt_probe_empty(void *stream);
//   int  dlrt_probe_wall_clock_khz(void);     rate of the constant counter, 0 if unknown
//   int  dlrt_probe_valu_ops_per_thread_iter(void);
// Return value: 0 on success, 1 if the launch failed.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.h"

namespace {

constexpr int kThreads = 256;
constexpr int kRows = 4, kCols = 8;  // 32 accumulators per lane: at most 64 registers, so 8 waves fit a SIMD

__global__ __launch_bounds__(kThreads) void valu_probe_kernel(uint64_t *clocks, uint32_t *sink, int iters)
{
    uint32_t a[kRows], w[kCols];
    int acc[kRows][kCols];
#pragma unroll
    for (int i = 0; i < kRows; ++i) a[i] = 0x9e3779b9u * (threadIdx.x + i + 1);
#pragma unroll
    for (int j = 0; j < kCols; ++j) w[j] = 0x85ebca6bu ^ (threadIdx.x * 7 + j);
#pragma unroll
    for (int i = 0; i < kRows; ++i)
#pragma unroll
        for (int j = 0; j < kCols; ++j) acc[i][j] = 0;

    const uint64_t c0 = clock64(), r0 = wall_clock64();
#pragma unroll 4
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kRows; ++i) {
            uint32_t t0, t1;
            asm volatile("v_and_b32 %8, %10, %11\n\t"
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
                         : "+v"(acc[i][0]), "+v"(acc[i][1]), "+v"(acc[i][2]), "+v"(acc[i][3]), "+v"(acc[i][4]),
                           "+v"(acc[i][5]), "+v"(acc[i][6]), "+v"(acc[i][7]), "=&v"(t0), "=&v"(t1)
                         : "v"(a[i]), "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]));
        }
    }
    const uint64_t c1 = clock64(), r1 = wall_clock64();

    int s = 0;
#pragma unroll
    for (int i = 0; i < kRows; ++i)
#pragma unroll
        for (int j = 0; j < kCols; ++j) s += acc[i][j];
    sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = (uint32_t)s;
    if (threadIdx.x == 0) {
        clocks[2 * (size_t)blockIdx.x] = c1 - c0;      // shader-clock cycles of the loop
        clocks[2 * (size_t)blockIdx.x + 1] = r1 - r0;  // the same interval on the constant-rate counter
    }
}

__global__ __launch_bounds__(kThreads) void copy_probe_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads) dst[i] = src[i];
}

__global__ void empty_probe_kernel() {}

}  // namespace

extern "C" {

int dlrt_probe_valu_ops_per_thread_iter(void) { return 2 * kRows * kCols; }

int dlrt_probe_valu(int blocks, int iters, uint64_t *clocks, uint32_t *sink, void *stream)
{
    if (blocks <= 0 || iters <= 0 || !clocks || !sink) return 1;
    hipLaunchKernelGGL(valu_probe_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream), clocks,
                       sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int dlrt_probe_gemm_clocks(const uint32_t *A, const uint32_t *W, int32_t *C, int M, int N, int K, int abits, int wbits,
                           uint64_t *clocks, void *stream)
{
    if (!A || !W || !C || !clocks || M <= 0 || N <= 0 || K <= 0 || M % 64 || N % 64 || K % 128) return 1;
    if (abits < 1 || abits > 4 || wbits < 1 || wbits > 4) return 1;
    dlrt::ContractArgs g{};
    g.A = A; g.W = W; g.M = M; g.N = N; g.Kw = K / 32;
    g.a_msb_neg = 0; g.w_msb_neg = 1;
    g.vec = 4;
    g.clocks = reinterpret_cast<unsigned long long *>(clocks);
    dlrt::FusedOut o{};
    o.acc = C;
    o.qbits = 1;
    const hipStream_t q = static_cast<hipStream_t>(stream);
    const dlrt_status st = abits == 1   ? dlrt::launch_contract_a1(g, o, wbits, false, false, q)
                           : abits == 2 ? dlrt::launch_contract_a2(g, o, wbits, false, false, q)
                           : abits == 3 ? dlrt::launch_contract_a3(g, o, wbits, false, false, q)
                                        : dlrt::launch_contract_a4(g, o, wbits, false, false, q);
    return st == DLRT_OK ? 0 : 1;
}

int dlrt_probe_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst || bytes == 0 || bytes % 16 != 0) return 1;
    hipLaunchKernelGGL(copy_probe_kernel, dim3(256 * 16), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int dlrt_probe_empty(void *stream)
{
    hipLaunchKernelGGL(empty_probe_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int dlrt_probe_wall_clock_khz(void)
{
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return 0;
    return khz;
}

}  // extern "C"
