// Latency-oriented bit-serial contraction for small problems (single conv layers at batch 1):
// one WAVE owns an output tile of (LY*TM) rows x 32 columns over a slice of the reduction, so a
// layer with a few thousand outputs still spreads over hundreds of waves.
//
// Same arithmetic as contract.hip (Section V of arXiv 2207.08820: accumulate popcount(W[i] & A[j])
// per plane pair, apply shifts and signs once at the end); what differs is the decomposition:
//   * no block-wide barrier in the reduction loop: every wave stages its own A / W chunk in its own
//     LDS region and only has to order its own LDS traffic;
//   * the waves of a block split the reduction (ksplit = 1..8 slices of whole 4-word steps) and add
//     their partial sums through LDS at the end;
//   * the epilogue is fused: scale / bias (Section IV, t_hat = t_bar * s), requantization and the
//     bitplane packing of the NEXT layer's activations happen on the accumulators in registers,
//     so a chained layer is one launch and the int32 tensor never has to touch HBM.
// A wave tile is always 32 columns wide (lane grid LX x LY = (32/TN) x (2*TN), lane (lx, ly) owns
// columns lx*TN + s and rows ly + LY*r): the TN result bits of a lane are adjacent bits of one
// packed output word, which an OR-reduction over the LX lanes of a row completes.
//
// Compiled once per activation bit width (-DDLRT_ABITS=1..4), like contract.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "contract_common.h"
#include "dlrt.h"
#include "launch.h"

#ifndef DLRT_ABITS
#error "compile with -DDLRT_ABITS=1..4"
#endif

namespace {

using dlrt::ContractArgs;
using dlrt::FusedOut;

template <int WB> struct WaveTN { static constexpr int value = WB <= 2 ? 4 : 2; };

// Operands are fetched through buffer resources: a 32-bit byte offset per lane instead of a 64-bit address,
// and a load at an offset beyond the tensor returns zeros without touching memory, which is how words beyond the
// reduction and taps outside the image become zero (one select on the offset instead of one per loaded word).
// A wave at batch 1 is alone on its SIMD, so every instruction of this address arithmetic is exposed time.
constexpr uint32_t kOutOfRange = 0x80000000u;  // beyond any tensor this kernel accepts (at most 2^31 bytes)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#if defined(__HIP_DEVICE_COMPILE__)
using BufferResource = __amdgpu_buffer_rsrc_t;
__device__ __forceinline__ BufferResource make_resource(const uint32_t *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(base), 0, bytes, 0x00020000);
}
// VEC words at byte offset `offset` into out[0 .. VEC - 1]
template <int VEC>
__device__ __forceinline__ void load_words(BufferResource r, uint32_t offset, uint32_t *out)
{
    if (VEC == 4) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, offset, 0, 0);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    } else if (VEC == 2) {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, offset, 0, 0);
        out[0] = v.x; out[1] = v.y;
    } else {
        out[0] = __builtin_amdgcn_raw_buffer_load_b32(r, offset, 0, 0);
    }
}
// a * b + c on operands below 2^24, b uniform over the wave: one full-rate instruction (a 32-bit multiply runs
// at a quarter of that rate)
__device__ __forceinline__ uint32_t mad24(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t d;
    asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(b), "v"(c));
    return d;
}
// a * b on full 32-bit operands, b uniform.  Kept out of the compiler's sight: left to itself it folds such a
// product and a following add into a 64-bit multiply-add whose addend's upper half is whatever register follows,
// and waits for that register's pending load.
__device__ __forceinline__ uint32_t mul32(uint32_t a, uint32_t b)
{
    uint32_t d;
    asm("v_mul_lo_u32 %0, %1, %2" : "=v"(d) : "v"(a), "s"(b));
    return d;
}
// the same on signed 24-bit operands
__device__ __forceinline__ int mad24s(int a, int b, int c)
{
    int d;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(b), "v"(c));
    return d;
}
#else
__device__ inline int mad24s(int a, int b, int c) { return a * b + c; }
__device__ inline uint32_t mul32(uint32_t a, uint32_t b) { return a * b; }
struct BufferResource { const uint32_t *base; };  // host pass of the single-source compile: never executed
__device__ inline BufferResource make_resource(const uint32_t *base, uint32_t) { return BufferResource{base}; }
template <int VEC>
__device__ inline void load_words(BufferResource, uint32_t, uint32_t *out) { for (int e = 0; e < VEC; ++e) out[e] = 0u; }
__device__ inline uint32_t mad24(uint32_t a, uint32_t b, uint32_t c) { return a * b + c; }
#endif

// OR of `v` over each aligned group of LX (8 or 16) consecutive lanes, left in every lane of the group.
// DPP lane swaps within a row of 16 lanes: the two quad permutations give every lane its quad's OR, the
// half-row mirror (lane i <-> 7 - i) then brings in the other quad of the group of 8, the row mirror
// (i <-> 15 - i) the other half of a group of 16.  No LDS round trip, unlike a shuffle.
template <int LX>
__device__ __forceinline__ uint32_t or_across(uint32_t v)
{
    static_assert(LX == 8 || LX == 16, "lane groups of 8 or 16");
    constexpr int kSwap1 = 0xB1;        // quad_perm [1, 0, 3, 2]
    constexpr int kSwap2 = 0x4E;        // quad_perm [2, 3, 0, 1]
    constexpr int kHalfMirror = 0x141;  // row_half_mirror
    constexpr int kMirror = 0x140;      // row_mirror
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kSwap1, 0xf, 0xf, false);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kSwap2, 0xf, 0xf, false);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kHalfMirror, 0xf, 0xf, false);
    if (LX == 16) v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kMirror, 0xf, 0xf, false);
    return v;
}

// One launch can carry two independent problems of the same bit widths (e.g. the two convolutions that
// read the same activations): blockIdx.y picks the problem.
// TN: output columns per lane (4 for 1- and 2-bit weights, 2 for wider ones; 2 also for narrow weights in the
// "half" tile of (64 / 16) * TM = 4 rows, for layers with so few rows that 8-row tiles leave most of the chip idle).
template <int AB, int WB, int TM, int VEC, bool BIPOLAR, bool CONV, int TN>
__global__ __launch_bounds__(512) void contract_wave_kernel(const dlrt::WavePair pair, const int ksplit)
{
    const int which = blockIdx.y;
    const int tile = blockIdx.x;
    // All arguments are fetched here, in one batch of scalar loads from one base address: left to itself the
    // compiler loads each field where it is first used, and a wave that is alone on its SIMD then waits out a
    // round trip to the scalar cache a dozen times before its first global load is even issued.
    const dlrt::WaveProblem &prob = pair.p[which];
    const ContractArgs g = prob.g;
    const FusedOut o = prob.o;
    const int steps_base = prob.steps_base, steps_rem = prob.steps_rem, tiles = prob.tiles;
    const uint32_t magicSubN = prob.magicSubN;
    const int subN = prob.subN, subM = prob.subM, die_bits = prob.die_bits, lc = prob.lc;
    asm volatile("" ::"s"(subN), "s"(subM), "s"(die_bits), "s"(lc), "s"(g.a_bytes), "s"(g.w_bytes), "s"(g.tapMul), "s"(g.tapShift), "s"(g.magicKW16));
    asm volatile("" ::"s"(tiles), "s"(magicSubN), "s"(g.A), "s"(g.W), "s"(g.M), "s"(g.N), "s"(g.Kw), "s"(g.a_msb_neg), "s"(g.w_msb_neg), "s"(g.H),
                 "s"(g.Wd), "s"(g.Cw), "s"(g.KH), "s"(g.KW), "s"(g.Ho), "s"(g.Wo), "s"(g.sh), "s"(g.sw), "s"(g.ph), "s"(g.pw),
                 "s"(g.magicCw), "s"(g.magicKW), "s"(g.magicHW), "s"(g.magicWo), "s"(o.acc), "s"(o.y), "s"(o.q),
                 "s"(o.packed), "s"(o.scale), "s"(o.bias), "s"(o.qbits), "s"(steps_base), "s"(steps_rem));
    if (tile >= tiles) return;  // the other problem of the pair has more tiles
    constexpr int LX = 32 / TN, LY = 64 / LX;
    constexpr int ROWS = LY * TM;     // rows of the wave tile; it is 32 columns wide
    constexpr int UA = 4 * AB * ROWS; // 16-byte units of one staged A chunk (4 steps x planes x rows)
    constexpr int UW = 4 * WB * 32;
    constexpr int NA = (UA + 63) / 64, NW = UW / 64;  // staging slots per lane
    constexpr int NG = TN * WB;

    extern __shared__ uint4 lds[];  // ksplit regions of UA + UW units; reused for the final reduction

    const int lane = threadIdx.x & 63;
    const int ks = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave index = reduction slice
    uint4 *const la = lds + ks * (UA + UW);
    uint4 *const lw = la + UA;
    const int lx = lane % LX, ly = lane / LX;
    // tile index -> (tileM, tileN).  Consecutive blocks go to the chip's 8 dies in turn, each with an L2 of its
    // own; where the tile grid divides, the low die_bits (3) bits of the index pick one of r x c parts of
    // the grid (c = 2^lc, r * c = 8) and the rest a tile inside it, so that a die fetches 1/c of the weights
    // and 1/r of the activations of the layer instead of all of both.  Without a split die_bits and lc are 0
    // and subN is the whole width: the same arithmetic gives the row-major order.
    const int die = tile & ((1 << die_bits) - 1), local = tile >> die_bits;
    const int lm = checked_div(local, subN, magicSubN), ln = local - lm * subN;
    const int tileM = (die >> lc) * subM + lm, tileN = (die & ((1 << lc) - 1)) * subN + ln;
    const int m0 = tileM * ROWS, n0 = tileN * 32;

    // this wave's slice of the reduction, in steps of 4 words.  The waves that start first (they are alone on
    // their SIMD until the block's later waves arrive) take the odd steps, so that the waves sharing a SIMD
    // finish together.
    const int s_begin = ks * steps_base + min(ks, steps_rem), s_end = s_begin + steps_base + (ks < steps_rem ? 1 : 0);

    // ---- staging slots: lane + 64 t; four consecutive lanes fetch the 64 contiguous bytes of one (row or
    // column, plane).  Rows / columns beyond the matrix are clamped (loaded, never stored).  The weights come
    // first: their addresses need no pixel arithmetic, so their first fetch is in flight while the activation
    // side is still decoding its output pixels (a lone wave waits out every latency in full). ----
    const BufferResource rW = make_resource(g.W, g.w_bytes), rA = make_resource(g.A, g.a_bytes);
    uint32_t offW[NW];  // byte offset of the slot's four words at reduction word 0
    int dstW[NW], k4W[NW];
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        const int s = lane + 64 * t;
        const int k4 = s & 3, rp = s >> 2, plane = rp % WB, col = rp / WB;
        // column c is read by lane lx = c / TN as its s = c % TN: place it so that lanes of
        // consecutive lx read consecutive 16-byte units
        dstW[t] = (k4 * WB + plane) * 32 + (col % TN) * LX + col / TN;
        k4W[t] = k4;
        offW[t] = ((uint32_t)(min(n0 + col, g.N - 1) * WB + plane) * (uint32_t)g.Kw + (uint32_t)(k4 * 4)) * 4u;
    }

    uint4 stageA[NA], stageW[NW];
    // Four words of one row (or column) and plane, VEC at a time; a group at or beyond the reduction's end reads
    // as zero.  k0: the reduction word the slot starts at; off: the byte offset of that word.
    auto fetch_row = [&](BufferResource r, uint32_t off, int k0, bool guard) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; e += VEC) {
            const uint32_t o4 = off + 4u * e;
            load_words<VEC>(r, guard && k0 + e >= g.Kw ? kOutOfRange : o4, w + e);
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    };
    auto fetchW = [&](int kbase) {
        const bool guard = kbase + 16 > g.Kw;  // uniform: all four steps inside the reduction need no guards
#pragma unroll
        for (int t = 0; t < NW; ++t) stageW[t] = fetch_row(rW, offW[t] + 4u * kbase, kbase + k4W[t] * 4, guard);
    };
    fetchW(s_begin * 4);

    // scale / bias of this lane's columns: fetched now so that their latency hides behind the reduction
    float sc[TN], bs[TN];
#pragma unroll
    for (int s = 0; s < TN; ++s) sc[s] = bs[s] = 0.0f;
    if (ks == 0 && o.scale) {
#pragma unroll
        for (int s = 0; s < TN; ++s) sc[s] = o.scale[min(n0 + lx * TN + s, g.N - 1)];
        if (o.bias) {
#pragma unroll
            for (int s = 0; s < TN; ++s) bs[s] = o.bias[min(n0 + lx * TN + s, g.N - 1)];
        }
    }

    // Activations.  GEMM: like the weights.  Convolution (implicit im2col, see contract.hip): the slot's output
    // pixel gives the byte offset of its tap (0, 0), which may lie outside the image (the sum wraps; a tap is only
    // read where it lies inside, and there the tap's own offset brings the sum back into the tensor).
    uint32_t offA[NA];
    int dstA[NA], k4A[NA], ih0[NA], iw0[NA];
    const uint32_t pixel_bytes = (uint32_t)(AB * g.Cw * 4);
#pragma unroll
    for (int t = 0; t < NA; ++t) {
        const int s = lane + 64 * t;
        const int slot = s < UA ? s : 0;
        const int k4 = slot & 3, rp = slot >> 2, plane = rp % AB, row = rp / AB;
        dstA[t] = s < UA ? (k4 * AB + plane) * ROWS + row : -1;
        k4A[t] = k4;
        const int m = min(m0 + row, g.M - 1);
        ih0[t] = 0;
        iw0[t] = 0;
        if (CONV) {
            const int hw = g.Ho * g.Wo;
            const int n = checked_div(m, hw, g.magicHW), rem = m - n * hw;
            const int oh = checked_div(rem, g.Wo, g.magicWo), ow = rem - oh * g.Wo;
            ih0[t] = (int)mad24((uint32_t)oh, (uint32_t)g.sh, (uint32_t)-g.ph);
            iw0[t] = (int)mad24((uint32_t)ow, (uint32_t)g.sw, (uint32_t)-g.pw);
            const uint32_t pixel00 = (uint32_t)mad24s(ih0[t], g.Wd, (int)mul32((uint32_t)n, (uint32_t)(g.H * g.Wd))) + (uint32_t)iw0[t];
            offA[t] = mul32(pixel00, pixel_bytes) + (uint32_t)(plane * g.Cw * 4);
        } else {
            offA[t] = ((uint32_t)(m * AB + plane) * (uint32_t)g.Kw + (uint32_t)(k4 * 4)) * 4u;
        }
    }

    // VEC words of one tap: reduction word kwd -> (tap, channel word) -> (kh, kw); zero beyond the reduction and
    // outside the image.  Both divisions are a 24-bit multiply and a shift with constants from the host (a plain
    // shift when Cw is a power of two): full-rate instructions where a multiply-high division takes quarter-rate
    // ones, and no branch between the cases.
    const uint32_t magicKW16 = g.magicKW16;  // exact for tap * KW < 65536 (checked by the launcher)
    auto tap_load = [&](int t, int kwd, uint32_t *out) {
        const int tap = (int)(mad24((uint32_t)kwd, g.tapMul, 0u) >> g.tapShift), c = mad24s(tap, -g.Cw, kwd);
        const int kh = (int)(mad24((uint32_t)tap, magicKW16, 0u) >> 16), kw = mad24s(kh, -g.KW, tap);
        const int ih = ih0[t] + kh, iw = iw0[t] + kw;
        const bool ok = kwd < g.Kw && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.Wd;
        const uint32_t delta = mad24(mad24((uint32_t)kh, (uint32_t)g.Wd, (uint32_t)kw), pixel_bytes, (uint32_t)c << 2);
        load_words<VEC>(rA, ok ? offA[t] + delta : kOutOfRange, out);
    };
    auto fetchA = [&](int kbase) {
        if (CONV) {
#pragma unroll
            for (int t = 0; t < NA; ++t) {
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; e += VEC) tap_load(t, kbase + k4A[t] * 4 + e, w + e);
                stageA[t] = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
        if (!CONV) {
            const bool guard = kbase + 16 > g.Kw;
#pragma unroll
            for (int t = 0; t < NA; ++t) stageA[t] = fetch_row(rA, offA[t] + 4u * kbase, kbase + k4A[t] * 4, guard);
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int t = 0; t < NA; ++t)
            if (dstA[t] >= 0) la[dstA[t]] = stageA[t];
#pragma unroll
        for (int t = 0; t < NW; ++t) lw[dstW[t]] = stageW[t];
        // the chunk is read back by other lanes of this wave only: order the wave's LDS traffic
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    int acc[TM][AB][NG];
    int rowpc[TM][AB];
#pragma unroll
    for (int r = 0; r < TM; ++r)
#pragma unroll
        for (int j = 0; j < AB; ++j) {
            rowpc[r][j] = 0;
#pragma unroll
            for (int n = 0; n < NG; ++n) acc[r][j][n] = 0;
        }

    if (s_begin < s_end) {
        fetchA(s_begin * 4);
        commit();
    }
    for (int c0 = s_begin; c0 < s_end; c0 += 4) {
        const int nst = min(4, s_end - c0);
        const bool more = c0 + 4 < s_end;
        if (more) {
            fetchW((c0 + 4) * 4);
            fetchA((c0 + 4) * 4);
        }

        uint4 av[2][TM][AB], wv[2][TN][WB];
        auto lds_load = [&](int b, int k4) {
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int j = 0; j < AB; ++j) av[b][r][j] = la[(k4 * AB + j) * ROWS + ly + LY * r];
#pragma unroll
            for (int s = 0; s < TN; ++s)
#pragma unroll
                for (int i = 0; i < WB; ++i) wv[b][s][i] = lw[(k4 * WB + i) * 32 + s * LX + lx];
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
                        if (BIPOLAR) popc_acc(rowpc[r][j], a);
                        and_popc_group<NG>(acc[r][j], a, w);
                    }
            }
        };
        lds_load(0, 0);
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
            if (k4 < nst) {
                if (k4 + 1 < 4) lds_load((k4 + 1) & 1, k4 + 1);  // step k4+1 may lie beyond nst: read, not used
                mac(k4 & 1);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) commit();
    }

    // ---- plane pairs -> one integer per output (signs and shifts of Section V's double sum);
    // (x ^ mask) - mask negates x when mask is -1 ----
    const int wneg = g.w_msb_neg ? -1 : 0, aneg = g.a_msb_neg ? -1 : 0;
    int total[TM][TN];
#pragma unroll
    for (int r = 0; r < TM; ++r)
#pragma unroll
        for (int s = 0; s < TN; ++s) {
            int sum = 0;
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
                sum += j + 1 < AB ? part : (part ^ aneg) - aneg;
            }
            total[r][s] = sum;
        }

    // ---- add the slices of the other waves (the sum is linear in the slices).  A wave leaves its partial sums
    // in its OWN staging region (it is done with it; nobody else ever touches it), so one barrier is enough, and
    // wave 0 fetches all of them before it adds any: up to seven independent rounds of LDS reads in flight
    // instead of a loop of dependent ones (a region beyond ksplit reads wave 0's own, and is not added). ----
    if (ksplit > 1) {
        if (ks > 0) {
            int *mine = reinterpret_cast<int *>(la) + lane;
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int s = 0; s < TN; ++s) mine[(r * TN + s) * 64] = total[r][s];
        }
        __syncthreads();
        if (ks > 0) return;
        int part[7][TM][TN];
#pragma unroll
        for (int k = 1; k < 8; ++k) {
            const int *theirs = reinterpret_cast<const int *>(lds + (k < ksplit ? k : 0) * (UA + UW)) + lane;
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int s = 0; s < TN; ++s) part[k - 1][r][s] = theirs[(r * TN + s) * 64];
        }
#pragma unroll
        for (int k = 1; k < 8; ++k)
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int s = 0; s < TN; ++s) total[r][s] += k < ksplit ? part[k - 1][r][s] : 0;
    }

    // ---- fused epilogue on the registers of wave 0.  A wave at batch 1 is alone on its SIMD, so every taken
    // branch and every LDS round trip here is exposed latency: the chained-layer case (only the packed
    // output) is straight-line code, and the OR across the lanes of a row goes through DPP lane swaps. ----
    const float qmax = (float)((1 << o.qbits) - 1);
    const int Cwo = (g.N + 31) / 32;
    bool live[TM][TN];
    uint32_t q[TM][TN];
#pragma unroll
    for (int r = 0; r < TM; ++r)
#pragma unroll
        for (int s = 0; s < TN; ++s) {
            live[r][s] = m0 + ly + LY * r < g.M && n0 + lx * TN + s < g.N;
            q[r][s] = 0;
        }
    if (o.acc) {
#pragma unroll
        for (int r = 0; r < TM; ++r)
#pragma unroll
            for (int s = 0; s < TN; ++s)
                if (live[r][s]) o.acc[(size_t)(m0 + ly + LY * r) * g.N + n0 + lx * TN + s] = total[r][s];
    }
    if (o.scale) {
        float y[TM][TN];
#pragma unroll
        for (int r = 0; r < TM; ++r)
#pragma unroll
            for (int s = 0; s < TN; ++s) {
                y[r][s] = __fmaf_rn((float)total[r][s], sc[s], bs[s]);
                const uint32_t v = (uint32_t)fminf(fmaxf(rintf(y[r][s]), 0.0f), qmax);
                q[r][s] = live[r][s] ? v : 0u;  // columns beyond N are the zero padding of the packed words
            }
        if (o.y) {
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int s = 0; s < TN; ++s)
                    if (live[r][s]) o.y[(size_t)(m0 + ly + LY * r) * g.N + n0 + lx * TN + s] = y[r][s];
        }
        if (o.q) {
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int s = 0; s < TN; ++s)
                    if (live[r][s]) o.q[(size_t)(m0 + ly + LY * r) * g.N + n0 + lx * TN + s] = (uint8_t)q[r][s];
        }
    }
    if (o.packed) {  // uniform: every lane takes part in the lane swaps
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if (p >= o.qbits) break;
#pragma unroll
            for (int r = 0; r < TM; ++r) {
                uint32_t word = 0;
#pragma unroll
                for (int s = 0; s < TN; ++s) word |= ((q[r][s] >> p) & 1u) << (lx * TN + s);
                word = or_across<LX>(word);
                const int m = m0 + ly + LY * r;
                if (lx == 0 && m < g.M) o.packed[((size_t)m * o.qbits + p) * Cwo + tileN] = word;
            }
        }
    }
}

template <int WB, int TM, int VEC, bool BIPOLAR, bool CONV, int TN = WaveTN<WB>::value>
dlrt_status launch(const ContractArgs *g, const FusedOut *o, int count, int ksplit, hipStream_t stream)
{
    constexpr int AB = DLRT_ABITS;
    if constexpr (TM * TN * AB * WB > 72) {
        return DLRT_ERR_SHAPE;  // never planned: too many accumulators per lane
    } else {
        constexpr int ROWS = (64 / (32 / TN)) * TM;
        constexpr int units = 4 * AB * ROWS + 4 * WB * 32;
        dlrt::WavePair pair{};
        int64_t tiles = 0;
        for (int i = 0; i < count; ++i) {
            pair.p[i].g = g[i];
            pair.p[i].o = o[i];
            const int steps = (g[i].Kw + 3) / 4;
            pair.p[i].steps_base = steps / ksplit;
            pair.p[i].steps_rem = steps % ksplit;
            const int64_t t = (int64_t)((g[i].M + ROWS - 1) / ROWS) * ((g[i].N + 31) / 32);
            if (t > 0x7fffffffLL) return DLRT_ERR_SHAPE;
            pair.p[i].tiles = (int)t;
            // split of the tile grid over the 8 dies: r x c = 8 with the least fetch among those that divide it
            const int64_t tm = (g[i].M + ROWS - 1) / ROWS, tn = (g[i].N + 31) / 32;
            int lc = -1;
            double best = 0;
            for (int l = 0; l <= 3; ++l) {
                const int c = 1 << l, r = 8 >> l;
                if (tm % r != 0 || tn % c != 0) continue;
                const double fetch = (double)c * g[i].M * AB + (double)r * g[i].N * WB;
                if (lc < 0 || fetch < best) { best = fetch; lc = l; }
            }
            pair.p[i].die_bits = lc < 0 ? 0 : 3;
            pair.p[i].lc = lc < 0 ? 0 : lc;
            const int64_t sn = lc < 0 ? tn : tn >> lc;  // a local index < t is divided by sn
            pair.p[i].subN = (int)sn;
            pair.p[i].subM = lc < 0 ? 0 : (int)(tm >> (3 - lc));
            pair.p[i].magicSubN = t * sn >= (1LL << 32) ? 1u : sn == 1 ? 0u : (uint32_t)(((1ULL << 32) + sn - 1) / sn);
            if (t > tiles) tiles = t;
        }
        const size_t lds_bytes = (size_t)ksplit * units * 16;
        return dlrt::enqueue(contract_wave_kernel<AB, WB, TM, VEC, BIPOLAR, CONV, TN>, dim3((unsigned)tiles, (unsigned)count),
                             dim3(64 * ksplit), lds_bytes, stream, pair, ksplit);
    }
}

template <int WB, int TM, bool BIPOLAR, bool CONV, int TN = WaveTN<WB>::value>
dlrt_status pick_vec(const ContractArgs *g, const FusedOut *o, int count, int ksplit, hipStream_t stream)
{
    int vec = g[0].vec;  // both problems of a pair are loaded with the narrower of their widths
    if (count > 1 && g[1].vec < vec) vec = g[1].vec;
    if (vec == 4) return launch<WB, TM, 4, BIPOLAR, CONV, TN>(g, o, count, ksplit, stream);
    if (vec == 2) return launch<WB, TM, 2, BIPOLAR, CONV, TN>(g, o, count, ksplit, stream);
    return launch<WB, TM, 1, BIPOLAR, CONV, TN>(g, o, count, ksplit, stream);
}

// tm: rows per lane (1, 2, 4), or 0 for the half tile of 4 rows (1- and 2-bit weights; wider ones have it as tm = 1)
template <int WB, bool BIPOLAR, bool CONV>
dlrt_status pick_tm(const ContractArgs *g, const FusedOut *o, int count, int tm, int ksplit, hipStream_t stream)
{
    if constexpr (WB <= 2) {
        if (tm == 0) return pick_vec<WB, 1, BIPOLAR, CONV, 2>(g, o, count, ksplit, stream);
    }
    if (tm == 0) return DLRT_ERR_SHAPE;
    if (tm == 4) return pick_vec<WB, 4, BIPOLAR, CONV>(g, o, count, ksplit, stream);
    if (tm == 2) return pick_vec<WB, 2, BIPOLAR, CONV>(g, o, count, ksplit, stream);
    return pick_vec<WB, 1, BIPOLAR, CONV>(g, o, count, ksplit, stream);
}

template <bool CONV>
dlrt_status pick_wbits(const ContractArgs *g, const FusedOut *o, int count, int wbits, bool bipolar, int tm, int ksplit,
                       hipStream_t stream)
{
    switch (wbits) {
    case 1:
        return bipolar ? pick_tm<1, true, CONV>(g, o, count, tm, ksplit, stream)
                       : pick_tm<1, false, CONV>(g, o, count, tm, ksplit, stream);
    case 2: return pick_tm<2, false, CONV>(g, o, count, tm, ksplit, stream);
    case 3: return pick_tm<3, false, CONV>(g, o, count, tm, ksplit, stream);
    case 4: return pick_tm<4, false, CONV>(g, o, count, tm, ksplit, stream);
    }
    return DLRT_ERR_BITS;
}

}  // namespace

namespace dlrt {

#define DLRT_CAT2(a, b) a##b
#define DLRT_CAT(a, b) DLRT_CAT2(a, b)

dlrt_status DLRT_CAT(launch_wave_a, DLRT_ABITS)(const ContractArgs *g, const FusedOut *o, int count, int wbits,
                                                 bool bipolar, bool conv, int tm, int ksplit, hipStream_t stream)
{
    return conv ? pick_wbits<true>(g, o, count, wbits, bipolar, tm, ksplit, stream)
                : pick_wbits<false>(g, o, count, wbits, bipolar, tm, ksplit, stream);
}

}  // namespace dlrt
