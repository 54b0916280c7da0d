// Bit-serial contraction kernels for gfx950: GEMM and implicit-im2col convolution.
//
// Section V of arXiv 2207.08820: with operands split into bitplanes, a dot product is
//     sum_i sum_j popcount(W[i] & A[j]) << (i + j).
// Here every (j, i) plane pair of every output owns an int32 accumulator that is fed by
// v_and_b32 + v_bcnt_u32_b32 (the popcount instruction adds into its third operand, so one
// AND and one BCNT per 32 reduction elements per plane pair is all the inner loop issues).
// The shifts and the signs of two's-complement MSB planes are applied once per output after
// the reduction.  Bipolar 1-bit weights use 2*popcount(A[j] & W) - popcount(A[j]).
//
// Tiling (wave64, 256 threads = 16 x 16 lanes): a lane owns TM x TN outputs, rows ty + 16*r and
// columns tx + 16*s, so a block owns (16*TM) x (16*TN) outputs.  For 2 to 4 bits TM*abits and TN*wbits
// are kept near 8, which keeps the accumulator count near 64 per lane and the LDS traffic per VALU
// instruction constant; 1-bit operands get 4 rows / columns per lane (8 measured 2-9 % slower: 128-wide
// tiles leave too few blocks and half-empty tiles on narrow problems).  Packed A / W tiles are staged through LDS in chunks of
// 16 words (512 reduction elements), double buffered, laid out [k4][plane][row] in 16-byte
// units so that the inner loop reads whole uint4 with compile-time offsets and neighbouring
// lanes read neighbouring 16-byte units.
//
// This file is compiled once per activation bit width (-DDLRT_ABITS=1..4) so that the
// instantiations build in parallel; contract_dispatch.hip picks the translation unit.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "contract_common.h"
#include "dlrt.h"
#include "launch.h"

#ifndef DLRT_ABITS
#error "compile with -DDLRT_ABITS=1..4"
#endif
// Two waves per SIMD: the other wave covers the LDS latency of a step, and the short live ranges let the
// register allocator keep everything else in registers (three waves per SIMD measured slower or spilled).
#define DLRT_WAVES_PER_EU 2

namespace {

using dlrt::ContractArgs;
using dlrt::FusedOut;

constexpr int kThreads = 256;
constexpr int kK4 = 4;   // 16-byte groups per chunk
constexpr int kKC = 16;  // words per chunk

// One 16-byte staging slot of a tile: which (row, plane, k4) of the chunk a thread moves.
template <int PLANES, int ROWS>
struct SlotMap {
    static constexpr int kSlots = kK4 * PLANES * ROWS;
    static constexpr int kPerThread = (kSlots + kThreads - 1) / kThreads;
    __device__ static void decode(int s, int &row, int &plane, int &k4)
    {
        // 8 consecutive lanes take 8 consecutive rows (one conflict-free 128-byte LDS write),
        // the next lane bits walk along K (one 64-byte global segment per row and plane).
        const int rowlo = s & 7;
        k4 = (s >> 3) & 3;
        const int rest = s >> 5;
        plane = rest % PLANES;
        row = (rest / PLANES) * 8 + rowlo;
    }
    __device__ static int lds_index(int row, int plane, int k4) { return (k4 * PLANES + plane) * ROWS + row; }
};

// VEC: widest aligned access, in words, that both operands allow (4, 2 or 1).  A template
// parameter rather than a run-time branch: the optimiser merges run-time variants of the same
// load into the narrowest one.
template <int AB, int WB, int TM, int TN, int VEC, bool BIPOLAR, bool CONV>
__global__ __launch_bounds__(kThreads, DLRT_WAVES_PER_EU) void contract_kernel(const ContractArgs g, const FusedOut o)
{
    constexpr int BM = 16 * TM, BN = 16 * TN;
    using MapA = SlotMap<AB, BM>;
    using MapW = SlotMap<WB, BN>;
    constexpr int kTileA = kK4 * AB * BM, kTileW = kK4 * WB * BN;  // uint4 units per buffer

    __shared__ uint4 ldsA[2 * kTileA];
    __shared__ uint4 ldsW[2 * kTileW];

#ifdef DLRT_CLOCK_PROBE
    const unsigned long long probe_c0 = clock64(), probe_r0 = wall_clock64();
#endif
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int tilesN = (g.N + BN - 1) / BN;
    int tileM, tileN;
    if (g.xcd_split) {
        // Consecutive blocks go to the chip's 8 dies (XCDs) in turn, each with an L2 of its own.  Block b is
        // therefore given a tile of die (b mod 8)'s own part of the tile grid, an r x c split of it with
        // r * c = 8 (c = 2^(xcd_split - 1), chosen by the launcher): every row band of A is then fetched from
        // HBM by c dies and every column band of W by r, instead of all of A by all eight.  4096^3 A2W2 with
        // 2 x 4: 24 MiB instead of 36 for the 8 MiB of operands.  Any mapping is correct (it is a bijection);
        // the launcher picks a split only among those that divide the grid evenly.
        const int lc = g.xcd_split - 1;
        const int tilesM = (g.M + BM - 1) / BM, subN = tilesN >> lc, subM = tilesM >> (3 - lc);
        const int die = blockIdx.x & 7, local = blockIdx.x >> 3;
        const int lm = local / subN, ln = local - lm * subN;
        tileM = (die >> lc) * subM + lm;
        tileN = (die & ((1 << lc) - 1)) * subN + ln;
    } else {
        tileM = blockIdx.x / tilesN;
        tileN = blockIdx.x - tileM * tilesN;
    }
    const int m0 = tileM * BM, n0 = tileN * BN;

    // ---- staging slots, resolved once.  Rows beyond the matrix are clamped to its last row:
    // they are loaded like any other and their outputs are never stored. ----
    const uint32_t *srcA[MapA::kPerThread];
    int dstA[MapA::kPerThread], k4A[MapA::kPerThread];
    int ih0[MapA::kPerThread], iw0[MapA::kPerThread];
#pragma unroll
    for (int t = 0; t < MapA::kPerThread; ++t) {
        const int s = tid + t * kThreads;
        int row, plane, k4;
        MapA::decode(s < MapA::kSlots ? s : 0, row, plane, k4);
        dstA[t] = s < MapA::kSlots ? MapA::lds_index(row, plane, k4) : -1;
        k4A[t] = k4;
        const int m = min(m0 + row, g.M - 1);
        ih0[t] = 0;
        iw0[t] = 0;
        if (CONV) {
            const int hw = g.Ho * g.Wo;
            const int n = checked_div(m, hw, g.magicHW), rem = m - n * hw;
            const int oh = checked_div(rem, g.Wo, g.magicWo), ow = rem - oh * g.Wo;
            ih0[t] = oh * g.sh - g.ph;
            iw0[t] = ow * g.sw - g.pw;
            // plane `plane` of pixel (n, 0, 0); pixel and channel-word offsets are added per load
            srcA[t] = g.A + (size_t)n * g.H * g.Wd * AB * g.Cw + plane * g.Cw;
        } else {
            srcA[t] = g.A + ((size_t)m * AB + plane) * g.Kw + k4 * 4;
        }
    }
    const uint32_t *srcW[MapW::kPerThread];
    int dstW[MapW::kPerThread], k4W[MapW::kPerThread];
#pragma unroll
    for (int t = 0; t < MapW::kPerThread; ++t) {
        const int s = tid + t * kThreads;
        int row, plane, k4;
        MapW::decode(s < MapW::kSlots ? s : 0, row, plane, k4);
        dstW[t] = s < MapW::kSlots ? MapW::lds_index(row, plane, k4) : -1;
        k4W[t] = k4;
        srcW[t] = g.W + ((size_t)min(n0 + row, g.N - 1) * WB + plane) * g.Kw + k4 * 4;
    }

    uint4 stageA[MapA::kPerThread], stageW[MapW::kPerThread];

    // implicit im2col: reduction word kwd = tap * Cw + c, tap = kh * KW + kw.  Loads VEC words of
    // one tap; a tap outside the image, or a word beyond the reduction, reads as zero.  Branch-free:
    // the address is clamped into the image and the result discarded.
    auto tap_load = [&](int t, int kwd, uint32_t *out) {
        bool ok = kwd < g.Kw;
        const int kc = ok ? kwd : 0;  // word 0 is always a valid, VEC-aligned stand-in
        const int tap = fast_div(kc, g.magicCw), c = kc - tap * g.Cw;
        const int kh = fast_div(tap, g.magicKW), kw = tap - kh * g.KW;
        const int ih = ih0[t] + kh, iw = iw0[t] + kw;
        ok = ok && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.Wd;
        const int ihc = min(max(ih, 0), g.H - 1), iwc = min(max(iw, 0), g.Wd - 1);
        const uint32_t *p = srcA[t] + (size_t)(ihc * g.Wd + iwc) * (AB * g.Cw) + c;
        if (VEC == 4) {
            const uint4 q = *reinterpret_cast<const uint4 *>(p);
            out[0] = ok ? q.x : 0u; out[1] = ok ? q.y : 0u; out[2] = ok ? q.z : 0u; out[3] = ok ? q.w : 0u;
        } else if (VEC == 2) {
            const uint2 q = *reinterpret_cast<const uint2 *>(p);
            out[0] = ok ? q.x : 0u; out[1] = ok ? q.y : 0u;
        } else {
            const uint32_t q = *p;
            out[0] = ok ? q : 0u;
        }
    };

    const int nchunks = (g.Kw + kKC - 1) / kKC, nfull = g.Kw / kKC;
    // 16-byte steps of the last chunk that hold any reduction words: a short or ragged reduction (a 1x1
    // conv over 64 channels is 2 words) does not pay for the zero padding of a whole chunk
    const int last_steps = (g.Kw - (nchunks - 1) * kKC + 3) / 4;
    auto fetch = [&](int chunk) {
        const int kbase = chunk * kKC;
        if (CONV) {
#pragma unroll
            for (int t = 0; t < MapA::kPerThread; ++t) {
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; e += VEC) tap_load(t, kbase + k4A[t] * 4 + e, w + e);
                stageA[t] = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
        if (chunk < nfull) {  // chunk wholly inside the reduction: no guards at all
            if (!CONV) {
#pragma unroll
                for (int t = 0; t < MapA::kPerThread; ++t) stageA[t] = load4<VEC>(srcA[t] + kbase);
            }
#pragma unroll
            for (int t = 0; t < MapW::kPerThread; ++t) stageW[t] = load4<VEC>(srcW[t] + kbase);
        } else {
            if (!CONV) {
#pragma unroll
                for (int t = 0; t < MapA::kPerThread; ++t)
                    stageA[t] = load4_tail<VEC>(srcA[t] + kbase, kbase + k4A[t] * 4, g.Kw);
            }
#pragma unroll
            for (int t = 0; t < MapW::kPerThread; ++t)
                stageW[t] = load4_tail<VEC>(srcW[t] + kbase, kbase + k4W[t] * 4, g.Kw);
        }
    };
    // Bipolar weights need popcount(A[j]) of every row (Section V's sum with weight bits 0 read as -1:
    // 2 * popcount(A & W) - popcount(A)).  It is counted where each activation word passes through a register
    // exactly once, in the thread that stages it: a partial count per staging slot (row, plane, 4-word column
    // of the chunk), summed over the four slots of a row and plane after the reduction.
    int stagepc[MapA::kPerThread];
#pragma unroll
    for (int t = 0; t < MapA::kPerThread; ++t) stagepc[t] = 0;
    auto commit = [&](int buf) {
#pragma unroll
        for (int t = 0; t < MapA::kPerThread; ++t)
            if (dstA[t] >= 0) {
                ldsA[buf * kTileA + dstA[t]] = stageA[t];
                if (BIPOLAR) stagepc[t] += __popc(stageA[t].x) + __popc(stageA[t].y) + __popc(stageA[t].z) + __popc(stageA[t].w);
            }
#pragma unroll
        for (int t = 0; t < MapW::kPerThread; ++t)
            if (dstW[t] >= 0) ldsW[buf * kTileW + dstW[t]] = stageW[t];
    };

    // acc[r][j][s * WB + i]: row r of the lane tile, activation plane j, column s, weight plane i
    constexpr int NG = TN * WB;
    int acc[TM][AB][NG];
#pragma unroll
    for (int r = 0; r < TM; ++r)
#pragma unroll
        for (int j = 0; j < AB; ++j)
#pragma unroll
            for (int n = 0; n < NG; ++n) acc[r][j][n] = 0;

    fetch(0);
    commit(0);
    __syncthreads();

    for (int chunk = 0; chunk < nchunks; ++chunk) {
        const int buf = chunk & 1;
        if (chunk + 1 < nchunks) fetch(chunk + 1);

        const uint4 *la = ldsA + buf * kTileA + ty;
        const uint4 *lw = ldsW + buf * kTileW + tx;
        // Four 16-byte steps per chunk, each reading its operands at its top.  The scheduling barrier
        // after each step keeps the compiler from hoisting every LDS read of the chunk to the top,
        // which would need four times the operand registers (and spills).
        uint4 av[1][TM][AB], wv[1][TN][WB];
        auto lds_load = [&](int b, int k4) {
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int j = 0; j < AB; ++j) av[b][r][j] = la[(k4 * AB + j) * BM + 16 * r];
#pragma unroll
            for (int s = 0; s < TN; ++s)
#pragma unroll
                for (int i = 0; i < WB; ++i) wv[b][s][i] = lw[(k4 * WB + i) * BN + 16 * s];
        };
        auto mac = [&](int b) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t w[NG];
#pragma unroll
                for (int s = 0; s < TN; ++s)
#pragma unroll
                    for (int i = 0; i < WB; ++i) {
                        const uint4 &q = wv[b][s][i];
                        w[s * WB + i] = e == 0 ? q.x : e == 1 ? q.y : e == 2 ? q.z : q.w;
                    }
#pragma unroll
                for (int r = 0; r < TM; ++r)
#pragma unroll
                    for (int j = 0; j < AB; ++j) {
                        const uint4 &q = av[b][r][j];
                        const uint32_t a = e == 0 ? q.x : e == 1 ? q.y : e == 2 ? q.z : q.w;
                        and_popc_group<NG>(acc[r][j], a, w);
                    }
            }
        };
        const int nsteps = chunk + 1 < nchunks ? kK4 : last_steps;  // block-uniform
#pragma unroll
        for (int k4 = 0; k4 < kK4; ++k4) {
            if (k4 < nsteps) {
                lds_load(0, k4);
                mac(0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        if (chunk + 1 < nchunks) commit(buf ^ 1);
        __syncthreads();
    }

    int rowpc[TM][AB];
    if (BIPOLAR) {
        __shared__ int pcbuf[BIPOLAR ? kK4 * AB * BM : 1];  // [k4][plane][row], as the staging slots are numbered
#pragma unroll
        for (int t = 0; t < MapA::kPerThread; ++t)
            if (dstA[t] >= 0) pcbuf[dstA[t]] = stagepc[t];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < TM; ++r)
#pragma unroll
            for (int j = 0; j < AB; ++j) {
                int n = 0;
#pragma unroll
                for (int k4 = 0; k4 < kK4; ++k4) n += pcbuf[(k4 * AB + j) * BM + ty + 16 * r];
                rowpc[r][j] = n;
            }
    }

    // ---- combine the plane pairs (signs and shifts of Section V's double sum), then the optional fused
    // epilogue of Section IV: scale / bias, requantization, and the bitplanes of the requantized result.
    // (x ^ mask) - mask negates x when mask is -1; the masks are uniform and live in scalar registers. ----
    const int wneg = g.w_msb_neg ? -1 : 0, aneg = g.a_msb_neg ? -1 : 0;
    auto combine = [&](int r, int s) {
        int total = 0;
#pragma unroll
        for (int j = 0; j < AB; ++j) {
            int part = 0;
            if (BIPOLAR) {
                part = 2 * acc[r][j][s] - rowpc[r][j];
            } else {
#pragma unroll
                for (int i = 0; i + 1 < WB; ++i) part += acc[r][j][s * WB + i] << i;
                const int msb = acc[r][j][s * WB + WB - 1] << (WB - 1);
                part += (msb ^ wneg) - wneg;
            }
            part <<= j;
            total += j + 1 < AB ? part : (part ^ aneg) - aneg;
        }
        return total;
    };

    const float qmax = (float)((1 << o.qbits) - 1);
    const int Cwo = (g.N + 31) / 32;
    const int wave_row = ty & 3;  // this lane's row among the four rows (ty values) of its wave
    float sc[TN], bs[TN];
    if (o.scale) {
#pragma unroll
        for (int s = 0; s < TN; ++s) {
            const int n = min(n0 + tx + 16 * s, g.N - 1);
            sc[s] = o.scale[n];
            bs[s] = o.bias ? o.bias[n] : 0.0f;
        }
    }
    // FULL: the tile lies wholly inside the output (block-uniform), so no element needs a bounds check;
    // which outputs exist is uniform too, so each is one scalar branch per tile row, not one per element
    auto write_tile = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (int r = 0; r < TM; ++r) {
            const int m = m0 + ty + 16 * r;
            const bool row_ok = FULL || m < g.M;
            bool ok[TN];
            int total[TN];
#pragma unroll
            for (int s = 0; s < TN; ++s) {
                ok[s] = FULL || (row_ok && n0 + tx + 16 * s < g.N);
                total[s] = combine(r, s);
            }
            const size_t row = (size_t)m * g.N + n0 + tx;  // element (m, n0 + tx); column s is 16 s further
            if (o.acc) {
#pragma unroll
                for (int s = 0; s < TN; ++s)
                    if (ok[s]) o.acc[row + 16 * s] = total[s];
            }
            uint32_t q[TN];
#pragma unroll
            for (int s = 0; s < TN; ++s) q[s] = 0;
            if (o.scale) {
                float y[TN];
#pragma unroll
                for (int s = 0; s < TN; ++s) {
                    y[s] = __fmaf_rn((float)total[s], sc[s], bs[s]);
                    if (ok[s]) q[s] = (uint32_t)fminf(fmaxf(rintf(y[s]), 0.0f), qmax);
                }
                if (o.y) {
#pragma unroll
                    for (int s = 0; s < TN; ++s)
                        if (ok[s]) o.y[row + 16 * s] = y[s];
                }
                if (o.q) {
#pragma unroll
                    for (int s = 0; s < TN; ++s)
                        if (ok[s]) o.q[row + 16 * s] = (uint8_t)q[s];
                }
            }
            if (o.packed) {  // block-uniform: every lane takes part in the ballots
                // A wave holds 4 rows x 16 columns per s: one ballot gives, for each of its rows, the 16-bit
                // field of columns 16 s .. 16 s + 15; two fields make one output word.
                for (int p = 0; p < o.qbits; ++p) {
#pragma unroll
                    for (int c = 0; c < TN / 2; ++c) {
                        const unsigned long long lo = __ballot((q[2 * c] >> p) & 1u), hi = __ballot((q[2 * c + 1] >> p) & 1u);
                        const uint32_t word = (uint32_t)((lo >> (16 * wave_row)) & 0xffffu) |
                                              ((uint32_t)((hi >> (16 * wave_row)) & 0xffffu) << 16);
                        if (tx == 0 && row_ok && (FULL || n0 + 32 * c < g.N))
                            o.packed[((size_t)m * o.qbits + p) * Cwo + n0 / 32 + c] = word;
                    }
                }
            }
        }
    };
    if (m0 + BM <= g.M && n0 + BN <= g.N) write_tile(std::true_type{});
    else write_tile(std::false_type{});
#ifdef DLRT_CLOCK_PROBE
    if (g.clocks && tid == 0) {
        g.clocks[2 * (size_t)blockIdx.x] = clock64() - probe_c0;
        g.clocks[2 * (size_t)blockIdx.x + 1] = wall_clock64() - probe_r0;
    }
#endif
}

template <int B> struct LaneTile { static constexpr int value = B <= 2 ? 4 : 2; };

template <int WB, int TM, int VEC, bool BIPOLAR, bool CONV>
dlrt_status launch_tile(const ContractArgs &g, const FusedOut &o, hipStream_t stream)
{
    constexpr int AB = DLRT_ABITS;
    constexpr int TN = LaneTile<WB>::value;
    const int64_t tilesM = (g.M + 16 * TM - 1) / (16 * TM), tilesN = (g.N + 16 * TN - 1) / (16 * TN);
    if (tilesM * tilesN > 0x7fffffffLL) return DLRT_ERR_SHAPE;
    // split of the tile grid over the 8 dies: r x c with the least HBM fetch, c * (bytes of A) + r * (bytes of W)
    ContractArgs ga = g;
    ga.xcd_split = 0;
    double best = 0;
    for (int lc = 0; lc <= 3; ++lc) {
        const int c = 1 << lc, r = 8 >> lc;
        if (tilesM % r != 0 || tilesN % c != 0) continue;
        const double fetch = (double)c * g.M * AB + (double)r * g.N * WB;  // per reduction word
        if (!ga.xcd_split || fetch < best) { best = fetch; ga.xcd_split = lc + 1; }
    }
    return dlrt::enqueue(contract_kernel<AB, WB, TM, TN, VEC, BIPOLAR, CONV>, dim3((unsigned)(tilesM * tilesN)),
                         dim3(kThreads), 0, stream, ga, o);
}

// Two tile heights per activation width: TM rows per lane (64-row tiles for 1 and 2 bits, 32-row tiles for 3 and
// 4), and half of that (twice as many blocks) for problems with few tiles; the launcher's plan says which.
template <int WB, int VEC, bool BIPOLAR, bool CONV>
dlrt_status launch(const ContractArgs &g, const FusedOut &o, hipStream_t stream)
{
    constexpr int TM = LaneTile<DLRT_ABITS>::value;
    if (g.half_rows) return launch_tile<WB, TM / 2, VEC, BIPOLAR, CONV>(g, o, stream);
    return launch_tile<WB, TM, VEC, BIPOLAR, CONV>(g, o, stream);
}

template <int WB, bool BIPOLAR, bool CONV>
dlrt_status pick_vec(const ContractArgs &g, const FusedOut &o, hipStream_t stream)
{
    if (g.vec == 4) return launch<WB, 4, BIPOLAR, CONV>(g, o, stream);
    if (g.vec == 2) return launch<WB, 2, BIPOLAR, CONV>(g, o, stream);
    return launch<WB, 1, BIPOLAR, CONV>(g, o, stream);
}

template <bool CONV>
dlrt_status pick_wbits(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar, hipStream_t stream)
{
    switch (wbits) {
    case 1: return bipolar ? pick_vec<1, true, CONV>(g, o, stream) : pick_vec<1, false, CONV>(g, o, stream);
    case 2: return pick_vec<2, false, CONV>(g, o, stream);
    case 3: return pick_vec<3, false, CONV>(g, o, stream);
    case 4: return pick_vec<4, false, CONV>(g, o, stream);
    }
    return DLRT_ERR_BITS;
}

}  // namespace

namespace dlrt {

#define DLRT_CAT2(a, b) a##b
#define DLRT_CAT(a, b) DLRT_CAT2(a, b)

dlrt_status DLRT_CAT(launch_contract_a, DLRT_ABITS)(const ContractArgs &g, const FusedOut &o, int wbits, bool bipolar,
                                                     bool conv, hipStream_t stream)
{
    return conv ? pick_wbits<true>(g, o, wbits, bipolar, stream) : pick_wbits<false>(g, o, wbits, bipolar, stream);
}

}  // namespace dlrt
