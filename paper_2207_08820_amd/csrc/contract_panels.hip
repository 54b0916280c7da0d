// Bit-serial contraction for LONG reductions with MANY rows: the convolution layers of a batched network
// (tens of thousands of output pixels, hundreds to thousands of reduction elements, 64 to 512 channels).
//
// Same arithmetic as the other contraction kernels (Section V of arXiv 2207.08820: popcount(W[i] & A[j]) per
// plane pair, shifts and signs applied once per output), decomposed for these shapes:
//   * a LANE owns one output row (pixel) and a WAVE 64 rows x NC output columns, a small unit of work: a layer
//     is tens of thousands of them, far more than the chip holds at once, so the hardware deals them out as
//     earlier ones finish and no compute unit is left with a large last tile (the tiled kernel lost 10 to 25 %
//     of these layers to that);
//   * the reduction is walked in PANELS of P packed words: the lane fetches its own P words of every
//     activation plane straight into registers (whole 16-byte pieces of one tap of its pixel: the im2col
//     matrix is never formed, not even in LDS), and they meet all NC columns before the next panel is fetched;
//   * the wave's weights, NC columns x all planes x the whole reduction (a contiguous piece of the packed
//     weight tensor, 4 to 9 KB), are copied once into the wave's own LDS region and read back as broadcasts
//     (every lane reads the same 16 bytes), 16 * abits VALU instructions per LDS read;
//   * one accumulator per (column, plane pair) lives across the panels; the fused epilogue (Section IV) runs
//     once per output and the lane assembles the NC result bits of each plane of ITS row into one or two bytes
//     of the next layer's packed activations.
// No block barrier, no lane-to-lane traffic: the only synchronisation is the wave's own LDS write -> read.
//
// Measured and dropped: splitting the reduction over 2 or 4 lane groups of a wave (32 or 16 rows per wave, partial
// sums added with lane exchanges), meant for layers with so few rows that a layer is only three waves per SIMD
// (a 7 x 7 layer over 4608 elements at batch 64): an LDS read then carries two or four different addresses
// instead of one broadcast, and the tap arithmetic moves from the scalar unit to the lanes; 0 to 5 % faster on
// two such layers, 5 to 40 % slower everywhere else.
//
// The activations are fetched with buffer loads: a tap outside the image, or a group beyond the reduction, is
// given an offset beyond the buffer's size, for which the hardware returns zeros without touching memory, so
// zero padding costs one select per 16-byte group instead of one per word, and the addresses are 32-bit.
//
// Limits (checked by the launcher, contract_dispatch.hip): reduction words a multiple of 4 and 16-byte aligned
// operands; for a convolution a whole number of 4-word groups per tap (channels a multiple of 128); activations
// of at most 2^31 bytes; NC * abits * wbits <= 64 accumulators.
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

constexpr int kMaxWaves = dlrt::kPanelMaxWaves;  // waves of a block that may share one tile's reduction

__device__ __forceinline__ uint32_t dot4(uint32_t a, uint32_t b, uint32_t c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_udot4(a, b, c, false);
#else
    (void)a; (void)b;
    return c;  // host pass of the single-source compile: never executed
#endif
}

// x with byte BYTE replaced by v rounded to nearest (ties to even) and saturated to [0, 255]: what
// v_cvt_pk_u8_f32 does in one instruction (negative values give 0).
template <int BYTE>
__device__ __forceinline__ uint32_t byte_from_float(float v, uint32_t x)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_cvt_pk_u8_f32(v, (uint32_t)BYTE, x);
#else
    return x | ((uint32_t)v << (8 * BYTE));
#endif
}

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

// acc += popcount(a & w) as one v_and_b32 + one accumulating v_bcnt_u32_b32; the empty asm keeps the chain of
// accumulating popcounts from being re-associated into separate counts and adds.
__device__ __forceinline__ void and_popc(int &acc, uint32_t a, uint32_t w)
{
    acc += __popc(a & w);
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(acc));
#endif
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Offset that lies beyond any buffer this kernel accepts (at most 2^31 bytes): a load there returns zeros.
constexpr uint32_t kOutOfRange = 0x80000000u;

// 16 bytes at byte offset `offset` of the buffer, zeros if the offset is out of range
#if defined(__HIP_DEVICE_COMPILE__)
using BufferResource = __amdgpu_buffer_rsrc_t;
__device__ __forceinline__ BufferResource make_resource(const uint32_t *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 load16(BufferResource r, uint32_t offset) { return __builtin_amdgcn_raw_buffer_load_b128(r, offset, 0, 0); }
#else
struct BufferResource { const uint32_t *base; };  // host pass of the single-source compile: never executed
__device__ inline BufferResource make_resource(const uint32_t *base, uint32_t) { return BufferResource{base}; }
__device__ inline u32x4 load16(BufferResource, uint32_t) { return u32x4{0u, 0u, 0u, 0u}; }
#endif

template <int AB, int WB, int NC, int P, bool BIPOLAR, bool CONV>
__global__ __launch_bounds__(64 * kMaxWaves) void contract_panel_kernel(const ContractArgs g, const FusedOut o, const int panels,
                                                                        const int kwaves /* waves of the block; divides panels */,
                                                                        const uint32_t magic_groups /* for division by panels / kwaves * P / 4 */)
{
    static_assert(P % 4 == 0 && NC % 8 == 0, "panels of whole 16-byte groups, whole output bytes");
    constexpr int G = P / 4;                 // 16-byte groups per panel and plane
    // The block's weights, zero beyond Kw / N: [panel][NC * WB][G] groups, so that within a panel every read is
    // the panel's base address plus a compile-time offset.  When several waves share the reduction, the partial
    // sums of waves 1 .. kwaves - 1 take the same memory after the last panel.
    extern __shared__ uint4 lds[];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform, and known to be
    const int kg = g.Kw >> 2;                // groups of the reduction
    const int my_panels = panels / kwaves, p_begin = wave * my_panels, p_end = p_begin + my_panels;
    const int kg_mine = my_panels * G;       // groups of this wave's panels (padded reduction)
    // block -> tile (row block, column group).  Consecutive blocks go to the chip's 8 dies in turn, each with an L2
    // of its own: die d takes the d-th eighth of the tiles in row-major order, so that the column groups of one row
    // block run on the same die one after the other (the rows' activations reach that die's L2 once) and the dies
    // get the same number of tiles to within one (dealing out whole row blocks left one die with 7 of 49 and the
    // others with 6: a sixth more time than work).
    const int col_groups = (g.N + NC - 1) / NC;
    const int64_t tiles = (int64_t)((g.M + 63) >> 6) * col_groups;
    const int die = blockIdx.x & 7;
    const int tile = (int)((tiles * die) >> 3) + (int)(blockIdx.x >> 3);
    if (tile >= (int)((tiles * (die + 1)) >> 3)) return;
    const int row_block = tile / col_groups, col_group = tile - row_block * col_groups;
    const int m = row_block * 64 + lane;
    const int mc = min(m, g.M - 1);          // rows beyond the matrix repeat the last row and are never stored
    const int n0 = col_group * NC;
    const bool row_ok = m < g.M;

    // ---- the wave's weights (its panels of every column and plane) -> LDS.  Columns n0 .. n0 + NC - 1 are one
    // contiguous run of the packed tensor, [column][plane][group]; group k of (column, plane) ci goes to panel
    // k / G, slot ci * G + k % G. ----
    {
        const uint4 *src = reinterpret_cast<const uint4 *>(g.W) + (size_t)n0 * WB * kg;
        const int cols = min(NC, g.N - n0);
        for (int u = lane; u < NC * WB * kg_mine; u += 64) {
            const int ci = fast_div(u, magic_groups), k = p_begin * G + (u - ci * kg_mine);  // (column, plane) pair, group of the padded reduction
            const bool ok = k < kg && ci < cols * WB;
            const uint4 q = src[ok ? ci * kg + k : 0];
            const int panel = k / G;
            lds[(panel * (NC * WB) + ci) * G + (k - panel * G)] = ok ? q : make_uint4(0u, 0u, 0u, 0u);
        }
        // read back by the other lanes of this wave only
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }

    // ---- where this lane's activations lie: byte offsets from the start of the tensor (32-bit), one buffer
    // resource per plane (plane j of a pixel or row lies j * plane_stride words after plane 0) ----
    const int plane_stride = CONV ? g.Cw : g.Kw;
    BufferResource planes[AB];
#pragma unroll
    for (int j = 0; j < AB; ++j) planes[j] = make_resource(g.A + j * plane_stride, g.a_bytes - 4u * j * plane_stride);
    int ih0 = 0, iw0 = 0;
    uint32_t lane_base;  // conv: the lane's image; GEMM: the lane's row
    if (CONV) {
        const int hw = g.Ho * g.Wo;
        const int img = checked_div(mc, hw, g.magicHW), rem = mc - img * hw;
        const int oh = checked_div(rem, g.Wo, g.magicWo), ow = rem - oh * g.Wo;
        ih0 = oh * g.sh - g.ph;
        iw0 = ow * g.sw - g.pw;
        lane_base = (uint32_t)img * (uint32_t)(g.H * g.Wd) * (uint32_t)(AB * g.Cw * 4);
    } else {
        lane_base = (uint32_t)mc * (uint32_t)(AB * g.Kw * 4);
    }
    const uint32_t pixel_bytes = AB * g.Cw * 4;
    // byte offset of the lane's tap (0, 0), which may lie outside the image (the sum wraps; only taps inside the
    // image are ever used, and for those the per-tap delta brings it back in range)
    uint32_t tap00 = lane_base + ((uint32_t)ih0 * (uint32_t)g.Wd + (uint32_t)iw0) * pixel_bytes;
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(tap00));  // kept as one value: a tap's offset is then one add, not the pixel arithmetic over again
#endif

    int acc[NC][AB][WB];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int j = 0; j < AB; ++j)
#pragma unroll
            for (int i = 0; i < WB; ++i) acc[c][j][i] = 0;
    int rowpc[AB];  // bipolar: popcount of the lane's row, per plane (Section V's sum with weight bit 0 read as -1)
#pragma unroll
    for (int j = 0; j < AB; ++j) rowpc[j] = 0;

    for (int p = p_begin; p < p_end; ++p) {
        // ---- this lane's P words of every activation plane; groups beyond the reduction and taps outside the
        // image read as zero (an out-of-range offset) ----
        uint32_t a[AB][P];
#pragma unroll
        for (int q = 0; q < G; ++q) {
            const int k = (p * G + q) * 4;      // first word of the group: uniform
            uint32_t offset;
            if (CONV) {
                const int kc = k < g.Kw ? k : 0;
                const int tap = fast_div(kc, g.magicCw), cw = kc - tap * g.Cw;
                const int kh = fast_div(tap, g.magicKW), kw = tap - kh * g.KW;  // all uniform: the scalar unit's work
                const int ih = ih0 + kh, iw = iw0 + kw;
                const bool ok = k < g.Kw && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.Wd;
                // (kh * W + kw) pixels and cw words further than tap (0, 0): a uniform delta, one add per lane
                const uint32_t delta = (uint32_t)(kh * g.Wd + kw) * pixel_bytes + 4u * cw;
                offset = ok ? tap00 + delta : kOutOfRange;
            } else {
                offset = k < g.Kw ? lane_base + 4u * k : kOutOfRange;
            }
#pragma unroll
            for (int j = 0; j < AB; ++j) {
                const u32x4 v = load16(planes[j], offset);
                a[j][4 * q] = v.x; a[j][4 * q + 1] = v.y; a[j][4 * q + 2] = v.z; a[j][4 * q + 3] = v.w;
            }
        }
        if (BIPOLAR) {
#pragma unroll
            for (int j = 0; j < AB; ++j)
#pragma unroll
                for (int k = 0; k < P; ++k) rowpc[j] += __popc(a[j][k]);
        }

        // ---- against every column and weight plane of the wave: the (column, plane)'s P words come from LDS as
        // broadcast reads, fetched one (column, plane) ahead of the one being multiplied ----
        const uint4 *wl = lds + p * (NC * WB * G);
        uint4 wbuf[2][G];
#pragma unroll
        for (int q = 0; q < G; ++q) wbuf[0][q] = wl[q];
#pragma unroll
        for (int ci = 0; ci < NC * WB; ++ci) {
            const int c = ci / WB, i = ci - c * WB;
            if (ci + 1 < NC * WB) {
#pragma unroll
                for (int q = 0; q < G; ++q) wbuf[(ci + 1) & 1][q] = wl[(ci + 1) * G + q];
            }
#pragma unroll
            for (int j = 0; j < AB; ++j)
#pragma unroll
                for (int q = 0; q < G; ++q) {
                    const uint4 &w = wbuf[ci & 1][q];
                    and_popc(acc[c][j][i], a[j][4 * q], w.x);
                    and_popc(acc[c][j][i], a[j][4 * q + 1], w.y);
                    and_popc(acc[c][j][i], a[j][4 * q + 2], w.z);
                    and_popc(acc[c][j][i], a[j][4 * q + 3], w.w);
                }
            __builtin_amdgcn_sched_barrier(0);  // one (column, plane) at a time: keeps the reads one step ahead, not sixteen
        }
    }

    // ---- several waves: the partial sums of the others meet in wave 0, which alone goes on.  (All waves of a
    // block share the row block, so the early exit above takes all of them or none.) ----
    if (kwaves > 1) {
        constexpr int SLOTS = NC * AB * WB + (BIPOLAR ? AB : 0);
        // [wave - 1][slot][lane], in place of the weights, which no wave reads any more once all have arrived
        int *red = reinterpret_cast<int *>(lds);
        __syncthreads();
        if (wave > 0) {
            int *mine = red + (wave - 1) * (SLOTS * 64) + lane;
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int j = 0; j < AB; ++j)
#pragma unroll
                    for (int i = 0; i < WB; ++i) mine[((c * AB + j) * WB + i) * 64] = acc[c][j][i];
            if (BIPOLAR) {
#pragma unroll
                for (int j = 0; j < AB; ++j) mine[(NC * AB * WB + j) * 64] = rowpc[j];
            }
        }
        __syncthreads();
        if (wave > 0) return;
        for (int w = 1; w < kwaves; ++w) {
            const int *theirs = red + (w - 1) * (SLOTS * 64) + lane;
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int j = 0; j < AB; ++j)
#pragma unroll
                    for (int i = 0; i < WB; ++i) acc[c][j][i] += theirs[((c * AB + j) * WB + i) * 64];
            if (BIPOLAR) {
#pragma unroll
                for (int j = 0; j < AB; ++j) rowpc[j] += theirs[(NC * AB * WB + j) * 64];
            }
        }
    }

    // ---- plane pairs -> one integer per output (signs and shifts of Section V's double sum) ----
    int wcoef[WB], acoef[AB];
#pragma unroll
    for (int i = 0; i < WB; ++i) wcoef[i] = (g.w_msb_neg && i == WB - 1) ? -(1 << i) : (1 << i);
#pragma unroll
    for (int j = 0; j < AB; ++j) acoef[j] = (g.a_msb_neg && j == AB - 1) ? -(1 << j) : (1 << j);
    int total[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        int t = 0;
#pragma unroll
        for (int j = 0; j < AB; ++j) {
            // plane 0 of an operand of two or more bits always weighs +1: it starts the sum without a multiply
            int part = BIPOLAR ? 2 * acc[c][j][0] - rowpc[j] : WB > 1 ? acc[c][j][0] : mad24(acc[c][j][0], wcoef[0], 0);
            if (!BIPOLAR) {
#pragma unroll
                for (int i = 1; i < WB; ++i) part = mad24(acc[c][j][i], wcoef[i], part);
            }
            t = (AB > 1 && j == 0) ? part : mad24(part, acoef[j], t);
        }
        total[c] = t;
    }

    // ---- fused epilogue (Section IV): y = fma(float(acc), scale, bias); q = clamp(rint(y), 0, 2^qbits - 1) ----
    const int cols = min(NC, g.N - n0);      // uniform
    const size_t out0 = (size_t)m * g.N + n0;
    if (o.acc && row_ok) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if (c < cols) o.acc[out0 + c] = total[c];
    }
    if (!o.scale) return;
    const float qmax = (float)((1 << o.qbits) - 1);
    uint32_t x[NC / 4];                      // q of column c in byte c % 4 of x[c / 4]
#pragma unroll
    for (int h = 0; h < NC / 4; ++h) x[h] = 0u;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int n = min(n0 + c, g.N - 1);
        const float y = __fmaf_rn((float)total[c], o.scale[n], o.bias ? o.bias[n] : 0.0f);
        if (o.y && row_ok && c < cols) o.y[out0 + c] = y;
        // rounding, the clamp at zero, the conversion and the byte insertion are one instruction; columns beyond N
        // give zero bits (the padding of the packed word)
        const float r = c < cols ? fminf(y, qmax) : 0.0f;
        x[c / 4] = c % 4 == 0 ? byte_from_float<0>(r, x[c / 4]) : c % 4 == 1 ? byte_from_float<1>(r, x[c / 4])
                 : c % 4 == 2 ? byte_from_float<2>(r, x[c / 4]) : byte_from_float<3>(r, x[c / 4]);
    }
    if (o.q && row_ok) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if (c < cols) o.q[out0 + c] = (uint8_t)(x[c / 4] >> (8 * (c % 4)));
    }
    if (o.packed && row_ok) {
        // bit p of columns 8h .. 8h + 7 is one byte of plane p's word: columns c and c + 4 share a byte of `nib`
        // (low and high nibble), and one dot product with {1, 2, 4, 8} gathers sum_c 2^c (bit(q_c) + 16 bit(q_c+4))
        const int Cwo = (g.N + 31) / 32;
        const bool last_group = n0 + NC >= g.N;
        for (int pl = 0; pl < o.qbits; ++pl) {
            uint8_t *dst = reinterpret_cast<uint8_t *>(o.packed + ((size_t)m * o.qbits + pl) * Cwo) + n0 / 8;
#pragma unroll
            for (int h = 0; h < NC / 8; ++h) {
                const uint32_t nib = x[2 * h] | (x[2 * h + 1] << 4);
                if (8 * h < cols) dst[h] = (uint8_t)dot4((nib >> pl) & 0x11111111u, 0x08040201u, 0u);
            }
            if (last_group) {  // the rest of the row's last word is padding: zero bits
                for (int b = n0 / 8 + (cols + 7) / 8; b < 4 * Cwo; ++b) dst[b - n0 / 8] = 0;
            }
        }
    }
}

template <int WB, int NC, int P, bool BIPOLAR, bool CONV>
dlrt_status launch_one(const ContractArgs &g, const FusedOut &o, int kwaves, hipStream_t stream)
{
    constexpr int AB = DLRT_ABITS;
    const int panels = (g.Kw + P - 1) / P;
    if (kwaves < 1 || kwaves > kMaxWaves || panels % kwaves != 0) return DLRT_ERR_SHAPE;
    // the block's weights over the padded reduction; later, in their place, the partial sums of the waves beyond the first
    const size_t w_bytes = (size_t)NC * WB * panels * P * 4, sum_bytes = (size_t)(kwaves - 1) * (NC * AB * WB + AB) * 64 * 4;
    const size_t lds_bytes = w_bytes > sum_bytes ? w_bytes : sum_bytes;
    if (lds_bytes > 65536) return DLRT_ERR_SHAPE;
    const int64_t bx = ((int64_t)g.M + 63) / 64, by = (g.N + NC - 1) / NC;
    const int64_t blocks = (bx * by + 7) / 8 * 8;  // the tiles, an eighth to each die
    if (blocks > 0x7fffffffLL) return DLRT_ERR_SHAPE;
    const uint32_t groups = (uint32_t)(panels / kwaves) * (P / 4);  // ceil(2^32 / groups), 0 standing for a divisor of 1
    const uint32_t magic_groups = groups == 1 ? 0u : (uint32_t)((0x100000000ULL + groups - 1) / groups);
    return dlrt::enqueue(contract_panel_kernel<AB, WB, NC, P, BIPOLAR, CONV>, dim3((unsigned)blocks), dim3(64 * kwaves),
                         lds_bytes, stream, g, o, panels, kwaves, magic_groups);
}

template <int WB, int NC, bool BIPOLAR, bool CONV>
dlrt_status pick_p(const ContractArgs &g, const FusedOut &o, int kwaves, hipStream_t stream)
{
    switch (dlrt::panel_words(g.Kw, kwaves)) {
    case 12: return launch_one<WB, NC, 12, BIPOLAR, CONV>(g, o, kwaves, stream);
    case 16: return launch_one<WB, NC, 16, BIPOLAR, CONV>(g, o, kwaves, stream);
    }
    return DLRT_ERR_SHAPE;  // no panel length that the waves share evenly
}

// ncols: 8, 16 or 32 columns per wave (NC * abits * wbits <= 64 accumulators)
template <int WB, bool BIPOLAR, bool CONV>
dlrt_status pick_panel(const ContractArgs &g, const FusedOut &o, int ncols, int kwaves, hipStream_t stream)
{
    constexpr int AB = DLRT_ABITS;
    if constexpr (AB * WB <= 2) {
        if (ncols == 32) return pick_p<WB, 32, BIPOLAR, CONV>(g, o, kwaves, stream);
    }
    if constexpr (AB * WB <= 4) {
        if (ncols == 16) return pick_p<WB, 16, BIPOLAR, CONV>(g, o, kwaves, stream);
    }
    if constexpr (AB * WB <= 8) {
        if (ncols == 8) return pick_p<WB, 8, BIPOLAR, CONV>(g, o, kwaves, stream);
    }
    return DLRT_ERR_SHAPE;  // never planned
}

template <bool CONV>
dlrt_status pick_wbits(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, int ncols, int kwaves, hipStream_t stream)
{
    switch (wbits) {
    case 1:
        return bipolar ? pick_panel<1, true, CONV>(g, o, ncols, kwaves, stream) : pick_panel<1, false, CONV>(g, o, ncols, kwaves, stream);
    case 2: return pick_panel<2, false, CONV>(g, o, ncols, kwaves, stream);
    case 3: return pick_panel<3, false, CONV>(g, o, ncols, kwaves, stream);
    case 4: return pick_panel<4, false, CONV>(g, o, ncols, kwaves, stream);
    }
    return DLRT_ERR_BITS;
}

}  // namespace

namespace dlrt {

#define DLRT_CAT2(a, b) a##b
#define DLRT_CAT(a, b) DLRT_CAT2(a, b)

dlrt_status DLRT_CAT(launch_panels_a, DLRT_ABITS)(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar,
                                                   bool conv, int ncols, int kwaves, hipStream_t stream)
{
    return conv ? pick_wbits<true>(g, o, wbits, bipolar, ncols, kwaves, stream)
                : pick_wbits<false>(g, o, wbits, bipolar, ncols, kwaves, stream);
}

}  // namespace dlrt
