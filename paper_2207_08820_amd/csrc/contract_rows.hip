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

// The longest register rows (16 and 18 words) are compiled for six resident waves per SIMD: left alone the compiler
// takes 108 registers (four waves) for its prologue's address arithmetic; at 80 nothing spills and the layers of
// 200704 x 64 x 576 and 50176 x 128 x 576 run 2 % faster (the last, thin round of waves is fuller).  Seven would spill.
template <int AB, int WB, int KW, bool BIPOLAR, bool CONV>
__global__ __launch_bounds__(kRowsPerBlock * kWavesPerBlock, (KW >= 16 && WB <= 2 ? 6 : 1)) void contract_rows_kernel(const ContractArgs g, const FusedOut o,
                                                                       const int ncols_full,
                                                                       const int fine_units /* per die, at most the fewest units a die has */,
                                                                       const uint32_t *__restrict__ Wp,
                                                                       const float *__restrict__ scale,
                                                                       const float *__restrict__ bias)
{
    // Wp / scale / bias repeat g.W / o.scale / o.bias as parameters of their own: only a read-only
    // pointer that provably aliases none of the stores is loaded through the scalar unit.
    // Wave -> unit (row block, column group).  Consecutive blocks go to the chip's 8 dies in turn, each with an L2
    // of its own: die d takes the d-th eighth of the units in row-major order, so that the column groups of one row
    // block run on the same die one after the other (the row's activations come from HBM once however the grid
    // divides) and the dies get the same number of units to within one.  The waves beyond a die's units leave here.
    const int col_groups = (g.N + ncols_full - 1) / ncols_full;
    const int64_t units = (int64_t)((g.M + kRowsPerBlock - 1) / kRowsPerBlock) * col_groups;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform, and known to be
    const int die = blockIdx.x & 7, local = (blockIdx.x >> 3) * kWavesPerBlock + wave;
    const int first = (int)((units * die) >> 3), mine = (int)((units * (die + 1)) >> 3) - first;
    // the die's last `fine_units` units are two waves of half the columns each, the others one wave: the blocks
    // handed out last are the small ones, and the launch's last round of waves a short one
    const int coarse = mine - fine_units, fine = local - coarse;
    if (fine >= 2 * fine_units) return;
    const int unit = first + (fine < 0 ? local : coarse + (fine >> 1));
    const int ncols = fine < 0 ? ncols_full : ncols_full >> 1;
    const int row_block = unit / col_groups, col_group = unit - row_block * col_groups;
    const int m = row_block * kRowsPerBlock + (threadIdx.x & 63);
    const int mc = min(m, g.M - 1);  // rows beyond the matrix are computed on the last row, never stored
    const int n0 = col_group * ncols_full + (fine < 0 ? 0 : (fine & 1) * ncols), n1 = min(n0 + ncols, g.N);

    // ---- this lane's activation row: abits planes of Kw words, zero beyond Kw.  For a convolution the
    // row is the im2col row of the lane's output pixel: word k is channel word c of tap (kh, kw), zero where
    // the tap lies outside the image (the address is clamped into the image and the word discarded). ----
    uint32_t a[AB][KW];
    int rowpc[AB];
#pragma unroll
    for (int j = 0; j < AB; ++j) rowpc[j] = 0;
    if (CONV) {
        const int hw = g.Ho * g.Wo;
        const int img = checked_div(mc, hw, g.magicHW), rem = mc - img * hw;
        const int oh = checked_div(rem, g.Wo, g.magicWo), ow = rem - oh * g.Wo;
        const int ih0 = oh * g.sh - g.ph, iw0 = ow * g.sw - g.pw;
        const uint32_t *image = g.A + (size_t)img * g.H * g.Wd * (AB * g.Cw);
        // One pixel's words, [plane][Cw], are contiguous.  When a tap is CW words wide and the reduction is a whole
        // number of taps, a tap is fetched as that one run with the widest loads its size allows, instead of a
        // 4-byte load per word: the lanes of a wave read 64 different pixels, so what a load instruction costs
        // the cache is its 64 separate lines, and the fewer instructions the better (measured: a 3x3 conv
        // over 64 channels took a third of its time in these loads).
        auto load_taps = [&](auto cw_tag) {
            constexpr int CW = decltype(cw_tag)::value, TAPS = KW / CW, RUN = AB * CW;
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const int kh = fast_div(t, g.magicKW), kw = t - kh * g.KW;  // uniform: the scalar unit's work
                const int ih = ih0 + kh, iw = iw0 + kw;
                const bool ok = (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.Wd;
                const int ihc = min(max(ih, 0), g.H - 1), iwc = min(max(iw, 0), g.Wd - 1);
                const uint32_t *pixel = image + (size_t)(ihc * g.Wd + iwc) * RUN;
                uint32_t v[RUN];
                if constexpr (RUN % 4 == 0) {  // the image base is 16-byte aligned, so every run of 4n words is
#pragma unroll
                    for (int e = 0; e < RUN; e += 4) {
                        const uint4 q = *reinterpret_cast<const uint4 *>(pixel + e);
                        v[e] = q.x; v[e + 1] = q.y; v[e + 2] = q.z; v[e + 3] = q.w;
                    }
                } else if constexpr (RUN % 2 == 0) {
#pragma unroll
                    for (int e = 0; e < RUN; e += 2) {
                        const uint2 q = *reinterpret_cast<const uint2 *>(pixel + e);
                        v[e] = q.x; v[e + 1] = q.y;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < RUN; ++e) v[e] = pixel[e];
                }
#pragma unroll
                for (int j = 0; j < AB; ++j)
#pragma unroll
                    for (int c = 0; c < CW; ++c) a[j][t * CW + c] = ok ? v[j * CW + c] : 0u;
            }
        };
        if (g.Kw == KW && g.Cw == 1) {
            load_taps(std::integral_constant<int, 1>{});
        } else if (g.Kw == KW && g.Cw == 2 && KW % 2 == 0) {
            load_taps(std::integral_constant<int, KW % 2 == 0 ? 2 : 1>{});
        } else if (g.Kw == KW && g.Cw == 4 && KW % 4 == 0) {
            load_taps(std::integral_constant<int, KW % 4 == 0 ? 4 : 1>{});
        } else if (g.Kw == KW && g.Cw == KW) {  // one tap (a strided 1x1 convolution)
            load_taps(std::integral_constant<int, KW>{});
        } else {
#pragma unroll
            for (int k = 0; k < KW; ++k) {
                const int kc = k < g.Kw ? k : 0;
                const int tap = fast_div(kc, g.magicCw), c = kc - tap * g.Cw;
                const int kh = fast_div(tap, g.magicKW), kw = tap - kh * g.KW;
                const int ih = ih0 + kh, iw = iw0 + kw;
                const bool ok = k < g.Kw && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.Wd;
                const int ihc = min(max(ih, 0), g.H - 1), iwc = min(max(iw, 0), g.Wd - 1);
                const uint32_t *pixel = image + (size_t)(ihc * g.Wd + iwc) * (AB * g.Cw) + c;
#pragma unroll
                for (int j = 0; j < AB; ++j) {
                    const uint32_t v = pixel[j * g.Cw];
                    a[j][k] = ok ? v : 0u;
                }
            }
        }
    } else {
        const uint32_t *arow = g.A + (size_t)mc * (AB * g.Kw);
        if (g.Kw == KW) {  // compile-time offsets: the row's AB * KW words are fetched with wide loads
#pragma unroll
            for (int j = 0; j < AB; ++j)
#pragma unroll
                for (int k = 0; k < KW; ++k) a[j][k] = arow[j * KW + k];
        } else {
#pragma unroll
            for (int j = 0; j < AB; ++j)
#pragma unroll
                for (int k = 0; k < KW; ++k) a[j][k] = k < g.Kw ? arow[j * g.Kw + k] : 0u;
        }
    }
    if (BIPOLAR) {
#pragma unroll
        for (int j = 0; j < AB; ++j)
#pragma unroll
            for (int k = 0; k < KW; ++k) rowpc[j] += __popc(a[j][k]);
    }

    // Plane weights with their signs (Section V's double sum): +-2^i, +-2^j, negative for the MSB plane of a
    // two's-complement operand.  Popcount sums stay below 2^10 and partial sums below 2^14 here, so the
    // combine is a chain of 24-bit multiply-adds (one full-rate instruction each).
    int wcoef[WB], acoef[AB];
#pragma unroll
    for (int i = 0; i < WB; ++i) wcoef[i] = (g.w_msb_neg && i == WB - 1) ? -(1 << i) : (1 << i);
#pragma unroll
    for (int j = 0; j < AB; ++j) acoef[j] = (g.a_msb_neg && j == AB - 1) ? -(1 << j) : (1 << j);
    // bipolar: sum_j 2^j (2 pc(A[j] & W) - pc(A[j])) = 2 sum_j 2^j pc(A[j] & W) - R with one constant R per row
    int neg_row_sum = 0;
#pragma unroll
    for (int j = 0; j < AB; ++j) neg_row_sum -= rowpc[j] << j;
    const float qmax = (float)((1 << o.qbits) - 1);
    const int Cwo = (g.N + 31) / 32;
    const bool row_ok = m < g.M;
    int lane_zero = 0;  // zero, but opaque to the compiler: an index with it is loaded per lane
#if defined(__HIP_DEVICE_COMPILE__)
    asm("v_mov_b32 %0, 0" : "=v"(lane_zero));
#endif
    const bool packed_only = !o.acc && !o.y && !o.q;  // the chained-layer case: nothing but the packed words

    // One output.  n is uniform over the wave, so the weight words, scale and bias come through
    // scalar loads and the AND takes them as scalar operands.  EXACT: the reduction has exactly KW words,
    // so every weight index is a compile-time offset from n * WB * KW and the loads of neighbouring
    // columns merge into wide scalar loads.
    // HORNER (unsigned activations): the activation planes of one weight plane share ONE accumulator, most
    // significant plane first, doubled between planes: the accumulating popcount then leaves
    // sum_j 2^j popcount(A[j] & W[i]) with one shift per further plane and no separate adds.  Two's-complement
    // activations (a negative MSB plane cannot be accumulated) take one accumulator per plane pair, on the
    // general path below, as does any call that wants more than the packed output.
    auto output = [&](int n, auto exact_tag, auto horner_tag) {
        constexpr bool EXACT = decltype(exact_tag)::value, HORNER = decltype(horner_tag)::value;
        const int kw = EXACT ? KW : g.Kw;
        const uint32_t *w = Wp + (size_t)n * (WB * kw);
        int total = 0;
        if (HORNER) {
#pragma unroll
            for (int i = 0; i < WB; ++i) {
                int acc = 0;
#pragma unroll
                for (int j = AB - 1; j >= 0; --j) {
                    if (j < AB - 1) acc <<= 1;
#pragma unroll
                    for (int k = 0; k < KW; ++k) {  // words beyond Kw: a[j][k] is zero, the weight index is clamped in bounds
                        acc += __popc(a[j][k] & w[i * kw + (EXACT || k < kw ? k : kw - 1)]);
                        keep_chain(acc);
                    }
                }
                total = BIPOLAR ? (acc << 1) + neg_row_sum : mad24(acc, wcoef[i], total);
            }
            return total;
        }
#pragma unroll
        for (int j = 0; j < AB; ++j) {
            int part = BIPOLAR ? -rowpc[j] : 0;
#pragma unroll
            for (int i = 0; i < WB; ++i) {
                int acc = 0;
#pragma unroll
                for (int k = 0; k < KW; ++k) {
                    acc += __popc(a[j][k] & w[i * kw + (EXACT || k < kw ? k : kw - 1)]);
                    keep_chain(acc);
                }
                part = BIPOLAR ? part + 2 * acc : mad24(acc, wcoef[i], part);
            }
            total = mad24(part, acoef[j], total);
        }
        return total;
    };

    uint32_t word[4] = {0u, 0u, 0u, 0u};
    auto add_bits = [&](int n, uint32_t q) {
        const int bit = n & 31;
#pragma unroll
        for (int p = 0; p < 4; ++p) word[p] |= ((q >> p) & 1u) << bit;
        if (bit == 31 || n == n1 - 1) {  // uniform: this row's word is complete (or the row ends)
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if (p < o.qbits && row_ok) o.packed[((size_t)m * o.qbits + p) * Cwo + (n >> 5)] = word[p];
                word[p] = 0u;
            }
        }
    };
    // min(y, qmax) with y = fma(float(acc), scale, bias): the upper clamp of the requantization, applied before the
    // rounding (the same number, qmax being an integer); byte_from_float() then rounds and clamps at zero.  With
    // no bias the product alone rounds to the same number as the fused multiply-add with +0 (up to the sign of a
    // zero, which the clamp removes).  A column's bias is the same for every lane but has to sit in a vector
    // register (an instruction reads at most one scalar register, and that is the scale): it comes through a
    // vector load of one address, which costs the VALUs nothing, instead of a register move per output.
    auto upper_clamped = [&](int total, int n, auto bias_tag) {
        constexpr bool HAS_BIAS = decltype(bias_tag)::value;
        const float y = HAS_BIAS ? __fmaf_rn((float)total, scale[n], bias[n + lane_zero]) : (float)total * scale[n];
        return fminf(y, qmax);
    };
    auto requantized = [&](int total, int n, auto bias_tag) { return clamp0(rintf(upper_clamped(total, n, bias_tag)), qmax); };
    auto packed_columns = [&](auto exact_tag, auto horner_tag, auto bias_tag) {
        // Eight columns at a time, in groups of CB with no branch inside a group: the scalar loads of a
        // group (weights, scale, bias) are issued together and waited for once, instead of one round trip
        // to the scalar cache per column.  The eight results land in the nibbles of four bytes (columns c and
        // c + 4 share a byte); bit p of every nibble is then one byte of plane p's word, gathered by ONE dot
        // product with the byte vector {1, 2, 4, 8}: sum_c 2^c (bit(q_c) + 16 bit(q_{c+4})).
        constexpr int CB = WB * KW <= 8 ? 4 : WB * KW <= 16 ? 2 : 1;
        int n = n0;
        for (; n + 8 <= n1; n += 8) {
            uint32_t x[2] = {0u, 0u};
#pragma unroll
            for (int c0 = 0; c0 < 8; c0 += CB) {
#pragma unroll
                for (int c = c0; c < c0 + CB; ++c) {
                    const float r = upper_clamped(output(n + c, exact_tag, horner_tag), n + c, bias_tag);
                    x[c >> 2] = (c & 3) == 0 ? byte_from_float<0>(r, x[c >> 2]) : (c & 3) == 1 ? byte_from_float<1>(r, x[c >> 2])
                              : (c & 3) == 2 ? byte_from_float<2>(r, x[c >> 2]) : byte_from_float<3>(r, x[c >> 2]);
                }
                __builtin_amdgcn_sched_barrier(0);  // keep the next group's scalar loads out of this group
            }
            const uint32_t nib = x[0] | (x[1] << 4);
            const int shift = n & 24;  // which byte of the 32-column word these eight columns are
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if (p < o.qbits) word[p] |= dot4((nib >> p) & 0x11111111u, 0x08040201u, 0u) << shift;
            }
            if (shift == 24 || n + 8 == n1) {
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    if (p < o.qbits && row_ok) {
                        uint32_t *dst = &o.packed[((size_t)m * o.qbits + p) * Cwo + (n >> 5)];
                        // a wave of 16 or 8 columns owns a half or a byte of the word (N is then a multiple of 32,
                        // so that every byte of every word has an owner)
                        if (ncols >= 32) *dst = word[p];
                        else if (ncols == 16) reinterpret_cast<uint16_t *>(dst)[(n >> 4) & 1] = (uint16_t)(word[p] >> (n & 16));
                        else reinterpret_cast<uint8_t *>(dst)[(n >> 3) & 3] = (uint8_t)(word[p] >> shift);
                    }
                    word[p] = 0u;
                }
            }
        }
        for (; n < n1; ++n)  // the last columns of a ragged N (whole-word waves only)
            add_bits(n, (uint32_t)requantized(output(n, exact_tag, horner_tag), n, bias_tag));
    };
    if (packed_only && !g.a_msb_neg) {
        // uniform over the launch; each combination is a loop of its own so that none pays for the others
        if (g.Kw == KW) {
            if (bias) packed_columns(std::true_type{}, std::true_type{}, std::true_type{});
            else packed_columns(std::true_type{}, std::true_type{}, std::false_type{});
        } else {
            if (bias) packed_columns(std::false_type{}, std::true_type{}, std::true_type{});
            else packed_columns(std::false_type{}, std::true_type{}, std::false_type{});
        }
    } else {
        for (int n = n0; n < n1; ++n) {
            const int total = output(n, std::false_type{}, std::false_type{});
            const size_t idx = (size_t)m * g.N + n;
            uint32_t q = 0;
            if (o.acc && row_ok) o.acc[idx] = total;
            if (scale) {
                const float y = __fmaf_rn((float)total, scale[n], bias ? bias[n] : 0.0f);
                q = (uint32_t)clamp0(rintf(y), qmax);
                if (o.y && row_ok) o.y[idx] = y;
                if (o.q && row_ok) o.q[idx] = (uint8_t)q;
            }
            if (o.packed) add_bits(n, q);
        }
    }
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

}  // namespace dlrt
