// Bit-serial contraction for SHORT reductions (at most 16 packed words, or 18): GEMMs over up to 512 elements,
// 1x1 convolutions over few channels, 3x3 convolutions over up to 64 channels (9 or 18 words), where the tiled
// kernels are mostly padding (their reduction step is 4 words, their tiles 32 or more columns wide, and
// their per-tile set-up outweighs the work).
//
// Same arithmetic as contract.hip (Section V of arXiv 2207.08820: popcount(W[i] & A[j]) per plane pair,
// shifts and signs applied once per output), decomposed the other way round: a LANE owns one output
// row.  It keeps the row's activation planes in registers (abits x KW words) and walks over the output
// columns; the weight words, scale and bias of a column are the same for every lane of the wave, so
// they are fetched with uniform (scalar) loads and feed the VALU as scalar operands: no LDS, no barrier,
// no lane-to-lane traffic.  The fused epilogue (Section IV: y = acc * scale + bias, requantization)
// runs per output, and the lane assembles the bitplane words of ITS row of the next layer's packed
// activations itself (eight results at a time, gathered with dot products as the packing kernel does), so
// the packed output needs no ballot or shuffle either.
//
// A wave covers 64 rows x `ncols` columns: a multiple of 32, so that waves own whole output words, or, on the
// packed-only path and when N fills whole words, 16 or 8, written as halves or bytes of the words (finer units
// for launches of only a few waves per SIMD).  The grid is one wave per (64 rows, ncols columns) unit, four to a
// block; every die gets an eighth of the units, and the last units of a launch of many rounds of waves may go out
// as two waves of half the columns each (planned_fine_units below).
// int32 / float / uint8 outputs are written one
// element per lane with a row stride between lanes: correct, but only the packed output is a fast path.
//
// Measured and dropped: software-pipelining the scalar loads (the next group's weights requested while this
// group is computed, both groups in scalar registers) was 0 to 7 % slower on 14 layer shapes; with seven waves
// per SIMD the other waves already cover a wave's wait for the scalar cache.  What is left between the
// kernel and its VALU floor is the per-output epilogue, the per-wave im2col prologue, and the start of the
// launch, where all waves (they fit the chip at once) fetch their rows before any of them computes.
//
// Compiled once per activation bit width (-DDLRT_ABITS=1..4), like contract.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "contract_common.h"
#include "dlrt.h"
#include "launch.h"

#ifndef DLRT_ABITS
#error "compile with -DDLRT_ABITS=1..4"
#endif

namespace {

using dlrt::ContractArgs;
using dlrt::FusedOut;

constexpr int kRowsPerBlock = 64;   // rows of one wave's tile: one per lane
// Waves per workgroup.  The waves of a block never synchronise or share anything; they only travel together
// because the chip hands out one-wave workgroups too slowly: with 6272 of them a 3x3 conv over 64 channels had
// 2.7 waves resident per SIMD on average although 6 fit, and a layer of 13 M outputs spent half of its 9 us
// being dispatched.
constexpr int kWavesPerBlock = 4;

__device__ __forceinline__ uint32_t dot4(uint32_t a, uint32_t b, uint32_t c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_udot4(a, b, c, false);
#else
    (void)a; (void)b;
    return c;  // host pass of the single-source compile: never executed
#endif
}

// Marks `acc` as opaque between two steps of a popcount chain: the accumulation then stays a chain of
// accumulating v_bcnt_u32_b32 (one instruction per word) instead of being re-associated into separate counts
// joined by three-input adds.  Emits no instruction.
__device__ __forceinline__ void keep_chain(int &acc)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(acc));
#else
    (void)acc;
#endif
}

// a * b + c on 24-bit operands, b uniform over the wave: one full-rate instruction (a general 32-bit
// multiply runs at a quarter of that rate).
__device__ __forceinline__ int mad24(int a, int b, int c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    int d;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(b), "v"(c));
    return d;
#else
    return a * b + c;
#endif
}

// clamp(x, 0, hi) in one instruction (x is finite here)
__device__ __forceinline__ float clamp0(float x, float hi)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_fmed3f(x, 0.0f, hi);
#else
    return fminf(fmaxf(x, 0.0f), hi);
#endif
}

// x with byte BYTE replaced by v converted to an 8-bit unsigned integer.  v_cvt_pk_u8_f32 rounds to nearest,
// ties to even, and saturates to [0, 255] (negative values and NaN give 0) - checked on the chip with ties,
// negatives, large values, infinities and NaN - so it is rint(), the lower clamp, the conversion and the byte
// insertion in ONE instruction; only the upper clamp remains for the caller.
template <int BYTE>
__device__ __forceinline__ uint32_t byte_from_float(float v, uint32_t x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_cvt_pk_u8_f32(v, (uint32_t)BYTE, x);
#else
    return x | ((uint32_t)v << (8 * BYTE));
#endif
}

// The work of one block of a problem (`block`: its index among that problem's blocks), for the two-problem kernel.
template <int AB, int WB, int KW, bool BIPOLAR, bool CONV>
__device__ __forceinline__ void rows_block(const ContractArgs g, const FusedOut o, const int ncols_full, const int fine_units,
                                           const uint32_t *__restrict__ Wp, const float *__restrict__ scale,
                                           const float *__restrict__ bias, const unsigned block)
{
#include "contract_rows_body.inc"
}

// The longest register rows (16 and 18 words) are compiled for six resident waves per SIMD: left alone the compiler
// takes 108 registers (four waves) for its prologue's address arithmetic; at 80 nothing spills and the layers of
// 200704 x 64 x 576 and 50176 x 128 x 576 run 2 % faster (the last, thin round of waves is fuller).  Seven would spill.
template <int AB, int WB, int KW, bool BIPOLAR, bool CONV>
__global__ __launch_bounds__(kRowsPerBlock * kWavesPerBlock, (KW >= 16 && WB <= 2 ? 6 : 1)) void contract_rows_kernel(const ContractArgs g, const FusedOut o,
                                                                       const int ncols_full, const int fine_units,
                                                                       const uint32_t *__restrict__ Wp,
                                                                       const float *__restrict__ scale,
                                                                       const float *__restrict__ bias)
{
    const unsigned block = blockIdx.x;
#include "contract_rows_body.inc"
}

// Two independent problems of the same bit widths and register-row length in one launch (two 1x1 convolutions of a
// single image, each too small to fill the chip and each a dependent launch of 3 us otherwise): the first
// `blocks0` blocks (a multiple of 8, so that the blocks of the second problem meet the dies as they would alone)
// are the first problem's.
template <int AB, int WB, int KW, bool BIPOLAR, bool CONV>
__global__ __launch_bounds__(kRowsPerBlock * kWavesPerBlock) void contract_rows_pair_kernel(
    const ContractArgs g0, const FusedOut o0, const int ncols0, const uint32_t *__restrict__ Wp0, const float *__restrict__ scale0,
    const float *__restrict__ bias0, const ContractArgs g1, const FusedOut o1, const int ncols1, const uint32_t *__restrict__ Wp1,
    const float *__restrict__ scale1, const float *__restrict__ bias1, const unsigned blocks0)
{
    if (blockIdx.x < blocks0) rows_block<AB, WB, KW, BIPOLAR, CONV>(g0, o0, ncols0, 0, Wp0, scale0, bias0, blockIdx.x);
    else rows_block<AB, WB, KW, BIPOLAR, CONV>(g1, o1, ncols1, 0, Wp1, scale1, bias1, blockIdx.x - blocks0);
}

// Whether waves of `ncols` columns exist for this call: whole output words, or, on the path that writes nothing but
// the packed output and only when N fills whole words (no ragged tail, no zero fill for anyone to own), 16 or 8
// columns, written as halves or single bytes of the words.
inline bool has_width(const ContractArgs &g, const FusedOut &o, int ncols)
{
    if (ncols >= 32) return ncols % 32 == 0;
    const bool packed_only = o.packed && !o.acc && !o.y && !o.q && !g.a_msb_neg;
    return (ncols == 8 || ncols == 16) && packed_only && g.N % 32 == 0;
}

// The last units of a die as waves of half the width.  A die holds `slots` waves at once (its compute units x the
// workgroups of this kernel that one holds x the waves of a workgroup), all of one length, so a launch runs in
// rounds: 1568 units on 768 slots are two full rounds and a third of 32 waves, which takes a whole wave's time at
// the low issue rate of a lone wave (measured: 200704 x 64 x 576 spends 5 % of its time there, 50176 x 128 x 576
// 9 %).  When the last round is at most a third full, its units - and as many again, for the dies and compute
// units do not fill evenly - go out as two waves of half the columns each: the short round takes half as long.
// Measured over tails of 1 to 13 times the remainder: flat within 1 % between 1.5 and 5 times.
inline int planned_fine_units(int64_t units, int resident, bool halves_exist)
{
    const int cus = dlrt::compute_units();
    if (!halves_exist || resident <= 0 || cus < 8) return 0;
    const int64_t slots = (int64_t)(cus / 8) * resident * kWavesPerBlock;
    const int64_t rest = units % slots;
    if (units < slots || rest == 0 || 3 * rest > slots) return 0;
    const int64_t fine = 2 * rest > slots / 8 ? 2 * rest : slots / 8;
    return (int)(fine < units ? fine : units);
}

// fine_units: how many of each die's (64 rows, ncols columns) units, the last ones, go out as two waves of half the
// columns each; -1: planned, -2: as many as every die has
template <int AB, int WB, int KW, bool BIPOLAR, bool CONV>
dlrt_status launch_one(const ContractArgs &g, const FusedOut &o, int ncols, int fine_units, hipStream_t stream)
{
    constexpr auto kernel = contract_rows_kernel<AB, WB, KW, BIPOLAR, CONV>;
    if (!has_width(g, o, ncols)) return DLRT_ERR_SHAPE;
    const int64_t bx = ((int64_t)g.M + kRowsPerBlock - 1) / kRowsPerBlock, by = (g.N + ncols - 1) / ncols;
    // per die: an eighth of the units, to within one; kWavesPerBlock waves to a block
    const int64_t most = (bx * by + 7) / 8, fewest = bx * by / 8;
    const bool halves_exist = ncols % 2 == 0 && has_width(g, o, ncols / 2);
    if (fine_units == -2) {
        if (!halves_exist) return DLRT_ERR_SHAPE;
        fine_units = (int)fewest;
    } else if (fine_units < 0) {
        fine_units = planned_fine_units(fewest, dlrt::resident_blocks<kernel>(kRowsPerBlock * kWavesPerBlock), halves_exist);
    }
    if (fine_units > fewest || (fine_units > 0 && !halves_exist)) return DLRT_ERR_SHAPE;
    const int64_t per_die = (most + fine_units + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t blocks = 8 * per_die;
    if (blocks * kWavesPerBlock > 0x7fffffffLL) return DLRT_ERR_SHAPE;
    return dlrt::enqueue(kernel, dim3((unsigned)blocks), dim3(kRowsPerBlock * kWavesPerBlock), 0, stream, g, o, ncols, fine_units,
                         g.W, o.scale, o.bias);
}

template <int AB, int WB, int KW, bool BIPOLAR>
dlrt_status launch_conv_or_gemm(const ContractArgs &g, const FusedOut &o, bool conv, int ncols, int fine_units, hipStream_t stream)
{
    return conv ? launch_one<AB, WB, KW, BIPOLAR, true>(g, o, ncols, fine_units, stream)
                : launch_one<AB, WB, KW, BIPOLAR, false>(g, o, ncols, fine_units, stream);
}

// Two GEMM-shaped problems (1x1 convolutions) with register rows of the same length in one launch.
template <int AB, int WB, int KW, bool BIPOLAR>
dlrt_status launch_pair(const ContractArgs g[2], const FusedOut o[2], const int ncols[2], hipStream_t stream)
{
    int64_t blocks[2];
    for (int i = 0; i < 2; ++i) {
        if (!has_width(g[i], o[i], ncols[i])) return DLRT_ERR_SHAPE;
        const int64_t bx = ((int64_t)g[i].M + kRowsPerBlock - 1) / kRowsPerBlock, by = (g[i].N + ncols[i] - 1) / ncols[i];
        blocks[i] = 8 * (((bx * by + 7) / 8 + kWavesPerBlock - 1) / kWavesPerBlock);
    }
    if ((blocks[0] + blocks[1]) * kWavesPerBlock > 0x7fffffffLL) return DLRT_ERR_SHAPE;
    return dlrt::enqueue(contract_rows_pair_kernel<AB, WB, KW, BIPOLAR, false>, dim3((unsigned)(blocks[0] + blocks[1])),
                         dim3(kRowsPerBlock * kWavesPerBlock), 0, stream, g[0], o[0], ncols[0], g[0].W, o[0].scale, o[0].bias,
                         g[1], o[1], ncols[1], g[1].W, o[1].scale, o[1].bias, (unsigned)blocks[0]);
}

// register-row length that a reduction of Kw words is compiled for (0: none)
inline int row_length(int Kw) { return Kw <= 1 ? 1 : Kw <= 2 ? 2 : Kw <= 4 ? 4 : Kw <= 8 ? 8 : Kw == 9 ? 9 : Kw <= 16 ? 16 : Kw == 18 ? 18 : 0; }

template <int AB, int WB, bool BIPOLAR>
dlrt_status pick_pair_kw(const ContractArgs g[2], const FusedOut o[2], const int ncols[2], hipStream_t stream)
{
    if (row_length(g[0].Kw) != row_length(g[1].Kw)) return DLRT_ERR_SHAPE;
    switch (row_length(g[0].Kw)) {  // (pairs exist for the short rows of 1x1 convolutions only)
    case 1: return launch_pair<AB, WB, 1, BIPOLAR>(g, o, ncols, stream);
    case 2: return launch_pair<AB, WB, 2, BIPOLAR>(g, o, ncols, stream);
    case 4: return launch_pair<AB, WB, 4, BIPOLAR>(g, o, ncols, stream);
    case 8: return launch_pair<AB, WB, 8, BIPOLAR>(g, o, ncols, stream);
    }
    return DLRT_ERR_SHAPE;
}

template <int AB, int WB, bool BIPOLAR>
dlrt_status pick_kw(const ContractArgs &g, const FusedOut &o, bool conv, int ncols, int fine_units, hipStream_t stream)
{
    if (g.Kw <= 1) return launch_conv_or_gemm<AB, WB, 1, BIPOLAR>(g, o, conv, ncols, fine_units, stream);
    if (g.Kw <= 2) return launch_conv_or_gemm<AB, WB, 2, BIPOLAR>(g, o, conv, ncols, fine_units, stream);
    if (g.Kw <= 4) return launch_conv_or_gemm<AB, WB, 4, BIPOLAR>(g, o, conv, ncols, fine_units, stream);
    if (g.Kw <= 8) return launch_conv_or_gemm<AB, WB, 8, BIPOLAR>(g, o, conv, ncols, fine_units, stream);
    if (g.Kw == 9) return launch_conv_or_gemm<AB, WB, 9, BIPOLAR>(g, o, conv, ncols, fine_units, stream);  // 3x3 taps of one word
    if (g.Kw <= 16) return launch_conv_or_gemm<AB, WB, 16, BIPOLAR>(g, o, conv, ncols, fine_units, stream);
    if (g.Kw == 18) return launch_conv_or_gemm<AB, WB, 18, BIPOLAR>(g, o, conv, ncols, fine_units, stream);  // 3x3 taps of two words
    return DLRT_ERR_SHAPE;  // never planned: the reduction is too long for a lane's registers
}

template <int AB>
dlrt_status pick_wbits(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, bool conv, int ncols,
                       int fine_units, hipStream_t stream)
{
    switch (wbits) {
    case 1:
        return bipolar ? pick_kw<AB, 1, true>(g, o, conv, ncols, fine_units, stream) : pick_kw<AB, 1, false>(g, o, conv, ncols, fine_units, stream);
    case 2: return pick_kw<AB, 2, false>(g, o, conv, ncols, fine_units, stream);
    case 3: return pick_kw<AB, 3, false>(g, o, conv, ncols, fine_units, stream);
    case 4: return pick_kw<AB, 4, false>(g, o, conv, ncols, fine_units, stream);
    }
    return DLRT_ERR_BITS;
}

}  // namespace

namespace dlrt {

#define DLRT_CAT2(a, b) a##b
#define DLRT_CAT(a, b) DLRT_CAT2(a, b)

dlrt_status DLRT_CAT(launch_rows_a, DLRT_ABITS)(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar,
                                                 bool conv, int ncols, int fine_units, hipStream_t stream)
{
    return pick_wbits<DLRT_ABITS>(g, o, wbits, bipolar, conv, ncols, fine_units, stream);
}

dlrt_status DLRT_CAT(launch_rows_pair_a, DLRT_ABITS)(const ContractArgs g[2], const FusedOut o[2], int wbits, bool bipolar,
                                                      const int ncols[2], hipStream_t stream)
{
    constexpr int AB = DLRT_ABITS;
    switch (wbits) {
    case 1: return bipolar ? pick_pair_kw<AB, 1, true>(g, o, ncols, stream) : pick_pair_kw<AB, 1, false>(g, o, ncols, stream);
    case 2: return pick_pair_kw<AB, 2, false>(g, o, ncols, stream);
    case 3: return pick_pair_kw<AB, 3, false>(g, o, ncols, stream);
    case 4: return pick_pair_kw<AB, 4, false>(g, o, ncols, stream);
    }
    return DLRT_ERR_BITS;
}

}  // namespace dlrt
