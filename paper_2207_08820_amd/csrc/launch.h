// Internal launch interface between the C ABI (api.hip) and the kernel files.  Arguments are
// already validated; every function enqueues on `stream` and reports only launch failures.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "dlrt.h"

namespace dlrt {

template <typename T> struct NonDeduced { using type = T; };

// Launches `kernel` and reports the status of THIS launch: hipLaunchKernel returns its own result, whereas
// hipGetLastError() after a <<<>>> launch would also pick up (and wrongly blame this call for) an error that an
// earlier, unrelated call of the process left behind.
template <typename... P>
dlrt_status enqueue(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                    typename NonDeduced<P>::type... args)
{
    void *argv[] = {const_cast<void *>(static_cast<const void *>(&args))...};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, argv, lds_bytes, stream);
    return e == hipSuccess ? DLRT_OK : DLRT_ERR_LAUNCH;
}

// How many workgroups of `threads` threads (and `lds_bytes` of dynamic LDS) of `Kernel` one compute unit holds at
// once, as the runtime computes it from the kernel's registers; the answer for the last (threads, lds_bytes) asked is
// kept per kernel, so a layer launched again and again asks once.  0: not known (the query failed), in which case
// callers plan as if they knew nothing about rounds of waves.
template <auto Kernel>
int resident_blocks(int threads, size_t lds_bytes = 0)
{
    static std::atomic<uint64_t> kept{0};   // (threads, lds_bytes, answer) in one word: 12 + 32 + 16 bits
    const uint64_t key = ((uint64_t)threads << 52) | ((uint64_t)(lds_bytes & 0xffffffffu) << 16);
    const uint64_t v = kept.load(std::memory_order_relaxed);
    if ((v & ~0xffffULL) == key && (v & 0xffff) != 0) return (int)(v & 0xffff);
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, Kernel, threads, lds_bytes) != hipSuccess || n <= 0) return 0;
    kept.store(key | (uint64_t)(n & 0xffff), std::memory_order_relaxed);
    return n;
}

// Compute units of the current device (256 on an MI355X, 32 per die), kept after the first call; 0: not known.
inline int compute_units()
{
    static std::atomic<int> kept{0};
    int v = kept.load(std::memory_order_relaxed);
    if (v > 0) return v;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 0;
    kept.store(v, std::memory_order_relaxed);
    return v;
}

// Optional outputs of the fused epilogue of both contraction kernels; any pointer may be null.
struct FusedOut {
    int32_t *acc;      // [M][N] accumulators
    float *y;          // [M][N] fma(float(acc), scale[n], bias[n])
    uint8_t *q;        // [M][N] clamp(rint(y), 0, 2^qbits - 1)
    uint32_t *packed;  // [M][qbits][ceil(N/32)] bitplanes of q (the next layer's packed activations)
    const float *scale, *bias;  // scale is required for y / q / packed
    int qbits;
};

// Arguments of one contraction launch (GEMM, or convolution as an implicit im2col GEMM).
struct ContractArgs {
    const uint32_t *A;  // GEMM: [M][abits][Kw]; conv: X [N][H][W][abits][Cw]
    const uint32_t *W;  // [N][wbits][Kw]
    int M, N, Kw;       // Kw: reduction words per plane (conv: KH*KW*Cw)
    int a_msb_neg, w_msb_neg;
    int vec;            // widest aligned load, in words, usable on both operands (4, 2 or 1)
    int half_rows;      // block kernel: tiles of half the usual height (32 instead of 64 rows, 16 instead of 32)
    int xcd_split;      // block kernel: 0, or 1 + log2(c) of the r x c split (r * c = 8) of the tile grid over the 8 dies
    uint32_t a_bytes;   // panel and per-wave kernels: size of the activation tensor in bytes (at most 2^31)
    uint32_t w_bytes;   // per-wave kernel: size of the weight tensor in bytes (at most 2^31)
    // Null in the library.  The benchmark's probe library builds the block kernel a second time with
    // DLRT_CLOCK_PROBE: each block then leaves here how many shader-clock cycles and how many ticks of the
    // constant-rate counter it lived ([2 * block], [2 * block + 1]), i.e. the clock the chip ran the kernel at.
    unsigned long long *clocks;
    // convolution geometry (unused by GEMM)
    int H, Wd, Cw, KH, KW, Ho, Wo, sh, sw, ph, pw;
    uint32_t magicCw, magicKW;  // ceil(2^32 / Cw), ceil(2^32 / KW); 0 stands for a divisor of 1
    uint32_t tapMul, tapShift;  // per-wave kernel: word / Cw = (word * tapMul) >> tapShift: (1, log2 Cw) for a power of two,
                                // else (ceil(2^16 / Cw), 16), exact while Kw * Cw < 2^16
    uint32_t magicKW16;         // ceil(2^16 / KW): tap / KW = (tap * magicKW16) >> 16 while tap * KW < 2^16
    uint32_t magicHW, magicWo;  // the same for Ho * Wo and Wo (output row -> image, pixel); 1: divide in hardware
};

// One translation unit per activation bit width (contract.hip with -DDLRT_ABITS=n).
dlrt_status launch_contract_a1(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, hipStream_t stream);
dlrt_status launch_contract_a2(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, hipStream_t stream);
dlrt_status launch_contract_a3(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, hipStream_t stream);
dlrt_status launch_contract_a4(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, hipStream_t stream);

// Kernel argument of the per-wave kernel: one problem, or two of the same bit widths in one launch.
// blockIdx.y names the problem, so a wave knows from its first instruction where its arguments lie; everything a
// problem needs sits in ONE struct so that the wave fetches it in a single batch of scalar loads from one base
// address (a lone wave pays every round trip to the scalar cache in full).  The grid is as wide as the larger
// problem and the surplus blocks of the smaller one leave at once.
struct WaveProblem {
    ContractArgs g;
    FusedOut o;
    int steps_base, steps_rem;  // 4-word steps per wave: base, and one more for the first `rem` waves
    int tiles;
    // tile index -> tile: the low die_bits bits pick one of r x c parts of the tile grid (c = 2^lc), the rest a
    // tile inside it, row-major over subN columns (die_bits = lc = 0, subN = ceil(N / 32): plain row-major order)
    int die_bits, lc, subN, subM;
    uint32_t magicSubN;  // for (tile >> die_bits) / subN; same convention as ContractArgs::magicHW
};
struct WavePair {
    WaveProblem p[2];
};

// Per-wave kernel (contract_wave.hip with -DDLRT_ABITS=n); g / o point at `count` (1 or 2) problems.
// tm = rows per lane (1, 2, 4), ksplit = waves per block that split the reduction (1, 2, 4, 8); both as
// planned by plan_wave().
dlrt_status launch_wave_a1(const ContractArgs *g, const FusedOut *o, int count, int wbits, bool bipolar, bool conv, int tm, int ksplit, hipStream_t stream);
dlrt_status launch_wave_a2(const ContractArgs *g, const FusedOut *o, int count, int wbits, bool bipolar, bool conv, int tm, int ksplit, hipStream_t stream);
dlrt_status launch_wave_a3(const ContractArgs *g, const FusedOut *o, int count, int wbits, bool bipolar, bool conv, int tm, int ksplit, hipStream_t stream);
dlrt_status launch_wave_a4(const ContractArgs *g, const FusedOut *o, int count, int wbits, bool bipolar, bool conv, int tm, int ksplit, hipStream_t stream);

// Row kernel (contract_rows.hip): one output row per lane, for reductions of at most 16 words, or of 18 (3x3
// taps of two words); GEMM or any convolution (a conv's words are those of its im2col row).  ncols: output
// columns per wave, a multiple of 32.
inline bool row_kernel_has(int Kw) { return Kw <= 16 || Kw == 18; }
dlrt_status launch_rows_a1(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols, int fine_units, hipStream_t stream);
dlrt_status launch_rows_a2(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols, int fine_units, hipStream_t stream);
dlrt_status launch_rows_a3(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols, int fine_units, hipStream_t stream);
dlrt_status launch_rows_a4(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols, int fine_units, hipStream_t stream);
// Two GEMM-shaped problems (1x1 convolutions) of the same bit widths and register-row length (1, 2, 4 or 8 words) in
// one launch; DLRT_ERR_SHAPE where no such kernel exists.
dlrt_status launch_rows_pair_a1(const ContractArgs g[2], const FusedOut o[2], int wbits, bool bipolar, const int ncols[2], hipStream_t stream);
dlrt_status launch_rows_pair_a2(const ContractArgs g[2], const FusedOut o[2], int wbits, bool bipolar, const int ncols[2], hipStream_t stream);
dlrt_status launch_rows_pair_a3(const ContractArgs g[2], const FusedOut o[2], int wbits, bool bipolar, const int ncols[2], hipStream_t stream);
dlrt_status launch_rows_pair_a4(const ContractArgs g[2], const FusedOut o[2], int wbits, bool bipolar, const int ncols[2], hipStream_t stream);

// Panel kernel (contract_panels.hip): one output row per lane, 64 rows x ncols columns per block, the reduction
// walked in panels of 12 or 16 words against weights held in LDS; for long reductions with many rows.  ncols is
// 8, 16 or 32 with ncols * abits * wbits <= 64 accumulators per lane.  kwaves (1 .. 4) waves of a block share the
// tile, each walking an equal number of panels, their partial sums added through LDS: smaller units of work for
// launches that are only a few waves per SIMD.  Needs Kw % 4 == 0 and 16-byte aligned
// operands (vec == 4), at most 64 KB of LDS per block, an activation tensor of at most 2^31 bytes (g.a_bytes),
// and for a convolution Cw % 4 == 0.
constexpr int kPanelMaxWaves = 4;

// Panel length for a reduction of Kw words shared by kwaves waves: 12 when the reduction is a whole number of
// 12-word panels and not of 16-word ones, else 16; the other length where only it gives a number of panels
// that the waves share evenly (and divides the reduction exactly).  0: neither does.
inline int panel_words(int Kw, int kwaves)
{
    const int first = Kw % 12 == 0 && Kw % 16 != 0 ? 12 : 16, second = 28 - first;
    if (kwaves < 1 || kwaves > kPanelMaxWaves) return 0;
    if (((Kw + first - 1) / first) % kwaves == 0) return first;
    if (Kw % second == 0 && (Kw / second) % kwaves == 0) return second;
    return 0;
}

inline bool panel_kernel_has(const ContractArgs &g, int abits, int wbits, bool conv, int ncols, int64_t a_bytes, int kwaves = 1)
{
    if (ncols != 8 && ncols != 16 && ncols != 32) return false;
    const int p = panel_words(g.Kw, kwaves);
    if (p == 0) return false;
    const int64_t padded = (int64_t)((g.Kw + p - 1) / p) * p;  // words per column and plane
    // the weights, and in their place after the last panel the partial sums of the waves beyond the first
    const int64_t lds_w = ncols * wbits * padded * 4, lds_sums = (int64_t)(kwaves - 1) * (ncols * abits * wbits + abits) * 256;
    const int64_t lds = lds_w > lds_sums ? lds_w : lds_sums;
    if (g.Kw % 4 != 0 || g.vec != 4 || ncols * abits * wbits > 64 || lds > 65536) return false;
    if (a_bytes > (1LL << 31)) return false;
    return !conv || g.Cw % 4 == 0;
}
dlrt_status launch_panels_a1(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols, int kwaves, hipStream_t stream);
dlrt_status launch_panels_a2(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols, int kwaves, hipStream_t stream);
dlrt_status launch_panels_a3(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols, int kwaves, hipStream_t stream);
dlrt_status launch_panels_a4(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols, int kwaves, hipStream_t stream);

// Conv geometry handed from the C ABI to the launcher.
struct ConvShape {
    int N, H, W, Cw, Co, KH, KW, Ho, Wo, sh, sw, ph, pw;
};

// GEMM / convolution with any subset of the fused outputs; the kernel (block or per-wave) is chosen by
// size.  tile_rows / ksplit are hints for the per-wave kernel (0 = planned); a non-zero hint forces it.
dlrt_status launch_gemm(const uint32_t *A, const uint32_t *W, int M, int N, int Kw, int abits, int wbits,
                        bool a_msb_neg, bool w_msb_neg, bool bipolar, const FusedOut &o, hipStream_t stream);

dlrt_status launch_conv(const uint32_t *X, const uint32_t *Wp, const ConvShape &c, int abits, int wbits,
                        bool a_msb_neg, bool w_msb_neg, bool bipolar, const FusedOut &o, int tile_rows, int ksplit,
                        hipStream_t stream);

// Two fused convolutions of the same bit widths in ONE launch of the per-wave kernel.
dlrt_status launch_conv_pair(const uint32_t *const X[2], const uint32_t *const Wp[2], const ConvShape c[2], int abits,
                             int wbits, bool a_msb_neg, bool w_msb_neg, bool bipolar, const FusedOut o[2],
                             hipStream_t stream);

// What launch_gemm / launch_conv would pick (no hints).
void query_plan(int M, int N, int Kw, int abits, int wbits, int *block_kernel, int *tile_rows, int *tile_cols, int *ksplit);

// rows x K elements (row stride ld) -> dst word (r, p, kw) at dst[r * row_stride + p * plane_stride + kw_off + kw].
// The generic destination strides let the same kernel emit both the [rows][bits][Kw] tensor and the
// per-tap padded layout of convolution weights.
struct PackArgs {
    const void *src;
    int src_type;          // dlrt_src
    int64_t rows, K, ld;
    int bits, enc;         // dlrt_encoding
    const float *scale;
    int scale_per_row;     // 0: one value; 1: one per row; 2: one per outer index (group of `taps` rows)
    uint32_t *dst;
    // destination addressing, in words
    int64_t taps;          // rows are grouped as [outer][taps]; 1 for plain tensors
    int64_t outer_stride;  // words between consecutive outer indices
    int64_t plane_stride;  // words between planes
    int64_t tap_stride;    // words between taps of one plane
};
dlrt_status launch_pack(const PackArgs &p, hipStream_t stream);

// int8 matrix-instruction GEMM on unpacked values (comparison variant); K % 16 == 0, 16-byte aligned rows.
dlrt_status launch_unpacked_gemm_i8(const int8_t *A, const int8_t *W, int32_t *C, int M, int N, int K,
                                    hipStream_t stream);

// 8-way dot-product GEMM on unpacked signed 4-bit values (comparison variant); K % 32 == 0, 16-byte aligned rows.
dlrt_status launch_unpacked_gemm_i4(const uint32_t *A, const uint32_t *W, int32_t *C, int M, int N, int K, hipStream_t stream);
dlrt_status launch_pack_nibbles(const int8_t *src, int64_t rows, int64_t K, uint32_t *dst, hipStream_t stream);

dlrt_status launch_epilogue(const int32_t *acc, const float *scale, const float *bias, int64_t rows, int C,
                            float *out_f32, uint8_t *out_q, int qbits, hipStream_t stream);

}  // namespace dlrt
