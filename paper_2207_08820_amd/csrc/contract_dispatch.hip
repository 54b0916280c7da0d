// Host-side set-up of a contraction launch: operand alignment, convolution geometry, the choice between
// the three contraction kernels (block kernel contract.hip, per-wave kernel contract_wave.hip, row kernel
// contract_rows.hip) and of their tiles, and the per-bit-width translation unit.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlrt.h"
#include "launch.h"

namespace {

// ceil(2^32 / d) for the kernels' multiply-high division; d = 1 would need 2^32 and is marked by 0.
uint32_t magic_for(int d) { return d == 1 ? 0u : (uint32_t)((0x100000000ULL + d - 1) / d); }

int widest_vec(const void *base, int64_t stride_words)
{
    const uintptr_t p = reinterpret_cast<uintptr_t>(base);
    if (p % 16 == 0 && stride_words % 4 == 0) return 4;
    if (p % 8 == 0 && stride_words % 2 == 0) return 2;
    return 1;
}

dlrt_status by_abits(const dlrt::ContractArgs &g, const dlrt::FusedOut &o, int abits, int wbits, bool bipolar,
                     bool conv, hipStream_t stream)
{
    switch (abits) {
    case 1: return dlrt::launch_contract_a1(g, o, wbits, bipolar, conv, stream);
    case 2: return dlrt::launch_contract_a2(g, o, wbits, bipolar, conv, stream);
    case 3: return dlrt::launch_contract_a3(g, o, wbits, bipolar, conv, stream);
    case 4: return dlrt::launch_contract_a4(g, o, wbits, bipolar, conv, stream);
    }
    return DLRT_ERR_BITS;
}

// The per-wave kernel addresses its operands with 32-bit byte offsets into buffer resources (loads beyond a
// tensor return zeros): both tensors must stay below 2^31 bytes.  Sizes in bytes, 0 if the kernel cannot take them.
bool wave_operand_bytes(const dlrt::ContractArgs &g, int abits, int wbits, bool conv, uint32_t *a_bytes, uint32_t *w_bytes)
{
    const int64_t wb = (int64_t)g.N * wbits * g.Kw * 4;
    int64_t ab = (int64_t)g.M * abits * g.Kw * 4;
    if (conv) {
        ab = (int64_t)g.M / ((int64_t)g.Ho * g.Wo) * g.H * g.Wd * abits * g.Cw * 4;
        // the tap arithmetic runs on 24-bit multiplies and a 16-bit reciprocal of KW
        if ((int64_t)g.KH * g.Wd + g.KW >= (1 << 24) || (int64_t)g.KH * g.KW * g.KW >= 65536 || abits * g.Cw * 4 >= (1 << 24))
            return false;
        if (g.Kw >= (1 << 24) || (g.tapShift == 16 && g.tapMul != 1 && (int64_t)g.Kw * g.Cw >= 65536)) return false;
    }
    if (ab > (1LL << 31) || wb > (1LL << 31)) return false;
    *a_bytes = (uint32_t)ab;
    *w_bytes = (uint32_t)wb;
    return true;
}

dlrt_status wave_by_abits(const dlrt::ContractArgs *g_in, const dlrt::FusedOut *o, int count, int abits, int wbits,
                          bool bipolar, bool conv, int tm, int ksplit, hipStream_t stream)
{
    dlrt::ContractArgs g[2];
    for (int i = 0; i < count; ++i) {
        g[i] = g_in[i];
        if (!wave_operand_bytes(g[i], abits, wbits, conv, &g[i].a_bytes, &g[i].w_bytes)) return DLRT_ERR_SHAPE;
    }
    switch (abits) {
    case 1: return dlrt::launch_wave_a1(g, o, count, wbits, bipolar, conv, tm, ksplit, stream);
    case 2: return dlrt::launch_wave_a2(g, o, count, wbits, bipolar, conv, tm, ksplit, stream);
    case 3: return dlrt::launch_wave_a3(g, o, count, wbits, bipolar, conv, tm, ksplit, stream);
    case 4: return dlrt::launch_wave_a4(g, o, count, wbits, bipolar, conv, tm, ksplit, stream);
    }
    return DLRT_ERR_BITS;
}

dlrt_status launch_rows(const dlrt::ContractArgs &g, const dlrt::FusedOut &o, int abits, int wbits, bool bipolar,
                        bool conv, int ncols, int fine_units, hipStream_t stream)
{
    switch (abits) {
    case 1: return dlrt::launch_rows_a1(g, o, wbits, bipolar, conv, ncols, fine_units, stream);
    case 2: return dlrt::launch_rows_a2(g, o, wbits, bipolar, conv, ncols, fine_units, stream);
    case 3: return dlrt::launch_rows_a3(g, o, wbits, bipolar, conv, ncols, fine_units, stream);
    case 4: return dlrt::launch_rows_a4(g, o, wbits, bipolar, conv, ncols, fine_units, stream);
    }
    return DLRT_ERR_BITS;
}

dlrt_status launch_panels(const dlrt::ContractArgs &g, const dlrt::FusedOut &o, int abits, int wbits, bool bipolar,
                          bool conv, int ncols, int kwaves, hipStream_t stream)
{
    switch (abits) {
    case 1: return dlrt::launch_panels_a1(g, o, wbits, bipolar, conv, ncols, kwaves, stream);
    case 2: return dlrt::launch_panels_a2(g, o, wbits, bipolar, conv, ncols, kwaves, stream);
    case 3: return dlrt::launch_panels_a3(g, o, wbits, bipolar, conv, ncols, kwaves, stream);
    case 4: return dlrt::launch_panels_a4(g, o, wbits, bipolar, conv, ncols, kwaves, stream);
    }
    return DLRT_ERR_BITS;
}

dlrt_status wave_by_abits(const dlrt::ContractArgs &g, const dlrt::FusedOut &o, int abits, int wbits, bool bipolar,
                          bool conv, int tm, int ksplit, hipStream_t stream)
{
    return wave_by_abits(&g, &o, 1, abits, wbits, bipolar, conv, tm, ksplit, stream);
}

// ---- tile planning -----------------------------------------------------------------------------
// Block kernel (contract.hip): lane tile {4,4,2,2}[bits] on 16 x 16 lanes.
int block_tile(int bits) { return 16 * (bits <= 2 ? 4 : 2); }

// The block kernel needs enough 256-thread blocks to give every compute unit one; below that the per-wave
// kernel spreads the same work over more, smaller waves.  Measured crossover on conv layers of 1568 .. 12544
// rows: about 100 tiles of 64 rows (200 blocks of the 32-row tile) for 1- and 2-bit activations; wider
// activations keep the earlier, untuned limit of 512 of their 32-row tiles.  The block kernel also needs its
// tiles filled: with N at most half a tile wide the per-wave kernel with its 32-column tiles measured 1.5 to
// 2.5 times faster at any number of rows.
int64_t wave_below(int abits) { return abits <= 2 ? 128 : 512; }

int64_t block_tiles(int M, int N, int abits, int wbits)
{
    return (int64_t)((M + block_tile(abits) - 1) / block_tile(abits)) * ((N + block_tile(wbits) - 1) / block_tile(wbits));
}

// Block kernel: every activation width has a full tile (64 rows for 1 and 2 bits, 32 rows for 3 and 4) and one
// of half that height.  With few tiles the half-height tile is 3 to 14 % faster on every conv-shaped problem
// measured (twice as many blocks fill the last round of resident blocks better and a tile's fixed cost is
// hidden behind more neighbours); with many tiles the full tile is as fast or up to 6 % faster (more reuse
// of each weight word read from LDS).  Measured crossovers, in full tiles: about 4096 for A2W2 and A2W1,
// between 1568 and 3136 for A3W3, none up to 12544 for A4W4.  A quarter-height tile measured slower than both.
bool prefer_half_rows(int M, int N, int abits, int wbits)
{
    const int64_t limit = abits <= 2 ? 4096 : abits == 3 ? 2048 : 16384;
    return block_tiles(M, N, abits, wbits) < limit;
}

bool prefer_wave_kernel(int M, int N, int abits, int wbits)
{
    // (also when M fills at most half a tile's rows: the same waste in the other direction)
    return block_tiles(M, N, abits, wbits) < wave_below(abits) || 2 * N <= block_tile(wbits) || 2 * M <= block_tile(abits);
}

struct WavePlan {
    int tm, ksplit;
    bool found;  // false: no feasible candidate matched the hints
};

// Per-wave kernel: wave tile (LY * tm) rows x 32 columns, LY = 8 for wbits <= 2 else 4.  Picks the
// (tm, ksplit) with the smallest modelled time: VALU and load cycles of one wave, stretched when
// there are more waves than the chip's 1024 SIMDs, plus the cost of the cross-wave reduction and a
// small charge for taller tiles.  Checked against a sweep of every (tile, split) on the GPU for the
// 26 distinct layer shapes of the two model-shaped stacks: the planned choice is within 1 % of the
// best in total and within 8 % on every single layer.
WavePlan plan_wave(int M, int N, int Kw, int abits, int wbits, int tile_rows_hint, int ksplit_hint)
{
    const int steps = (Kw + 3) / 4;
    WavePlan best{1, 1, false};
    double best_cost = 1e300;
    // tm = 0: the half tile of 4 rows x 32 columns that narrow weights have besides their 8-row one (2 columns per
    // lane instead of 4).  Half the work per wave and twice the tiles: it pays where the 8-row tiles are so few that
    // most compute units would stay idle while a few run all the waves of a deep reduction (a 7 x 7 layer over 512
    // channels is 112 tiles of 8 rows, each split over 8 waves on ONE compute unit).  Only then, or by hint.
    const bool few_tiles = (int64_t)((M + 7) / 8) * ((N + 31) / 32) <= 128;
    for (int tm = wbits <= 2 ? 0 : 1; tm <= 4; tm = tm ? tm * 2 : 1) {
        const int tn = wbits <= 2 && tm > 0 ? 4 : 2, ly = 2 * tn, tmv = tm ? tm : 1;
        if (tmv * tn * abits * wbits > 72) break;
        const int rows = ly * tmv;
        if (tile_rows_hint > 0 && rows != tile_rows_hint) continue;
        if (tm == 0 && tile_rows_hint == 0 && !few_tiles) continue;
        const int64_t tiles = (int64_t)((M + rows - 1) / rows) * ((N + 31) / 32);
        for (int ks = 1; ks <= 8; ks *= 2) {
            if (ksplit_hint > 0 && ks != ksplit_hint) continue;
            if (ks > 1 && ks > steps) break;
            const int units = 4 * abits * rows + 4 * wbits * 32;
            if ((int64_t)ks * units * 16 > 65536) break;
            const int spw = (steps + ks - 1) / ks;
            // a lone wave keeps a SIMD about 70 % busy; with several waves per SIMD they cover each other
            const double over = (double)tiles * ks / 1024;
            // With more waves than SIMDs a wave's own cost (addresses, the exchange of partial sums: about a thousand
            // issue cycles) is no longer hidden behind idle SIMDs, and a split down to one or two steps per wave adds
            // more of it than it saves: 400 x 512 x 512 at A2W2 and A4W1 measured 4.2 us unsplit, 5.0 in two, 6.6 in four.
            if (ks > 1 && over > 1 && spw < 3 && ksplit_hint == 0) break;
            const double eff = over <= 1 ? 0.7 : (0.7 + 0.12 * (over - 1) < 0.95 ? 0.7 + 0.12 * (over - 1) : 0.95);
            const double valu = (double)spw * 4 * tmv * tn * abits * wbits * 2 * 4 / eff;
            const double load = (double)spw * (abits * rows + wbits * 32) * 16 / 32;
            const double cost = (valu + load) * (over > 1 ? over : 1.0) + (ks > 1 ? 500 + 120 * ks : 0) + (tmv - 1) * 150;
            if (cost < best_cost) { best_cost = cost; best = WavePlan{tm, ks, true}; }
        }
    }
    return best;
}

// The row kernel (one output row per lane, whole reduction in registers, weights through scalar loads) has no
// per-tile set-up, LDS traffic or barrier, so on short reductions it beats the tiled kernels as soon as
// there are enough waves of 64 rows x 32 columns to fill the chip; how many depends on how well the
// reduction fits the tiled kernels' 4- and 16-word steps.  Measured on convolutions of 3136 .. 200704 output
// pixels x 32 .. 512 channels at A1W1, A2W1, A2W2, A3W2 and A4W4: from the wave counts below on it is as fast
// or (mostly) 1.1 to 4 times faster than the better of the other two, below them slower.  An 18-word
// reduction (3x3 taps over 64 channels) needs 18 x wbits scalar registers of weights per column, which only
// pays for 1- and 2-bit weights (A4W4 measured half the block kernel's speed).
int64_t row_kernel_waves(int64_t M, int N) { return ((M + 63) / 64) * ((N + 31) / 32); }

// `halves`: the call may use waves of 8 or 16 columns (nothing but the packed output, unsigned activations, whole
// output words).  Such waves fill the chip at a quarter of the rows, which moves the row kernel's territory down to
// single images: from 800 waves of 8 columns on it measured 5 to 25 % faster than the tiled kernels on every
// layer tried with a reduction of up to 9 words, or 18 (6400 .. 25600 pixels x 32 .. 128 channels, A2W1), slower
// below (1600 pixels x 128 channels, 3136 x 64 at 18 words).
bool prefer_rows_kernel(int64_t M, int N, int Kw, int abits, int wbits, bool halves)
{
    // (18 words: 1- and 2-bit weights, or 2-bit activations with 4-bit weights, which measured 24 to 38 % ahead of the
    // block kernel on two layers of 50176 and 200704 pixels; A3W3 and A4W4 stay behind it)
    if (!dlrt::row_kernel_has(Kw) || (Kw > 16 && wbits > 2 && abits * wbits > 8)) return false;
    if (M < 2048) return false;  // lanes idle on few rows (none measured below 3136)
    if (((M + 63) / 64 + 7) * ((N + 7) / 8) > 0x7fffffffLL) return false;  // more blocks than a grid holds
    if (halves && N % 32 == 0 && (Kw <= 9 || (Kw == 18 && abits <= 2)) && ((M + 63) / 64) * (N / 8) >= 800) return true;
    const int64_t from = Kw == 1 ? 256 : Kw == 2 ? 384 : Kw <= 4 ? 1024 : Kw <= 9 ? 1536 : Kw <= 16 ? 12288 : 3072;
    return row_kernel_waves(M, N) >= from;
}

// The panel kernel (one output row per lane, 64 rows x 8 columns per wave, the reduction walked in panels against
// weights in LDS) has small units of work that the hardware deals out as earlier ones finish, where the block
// kernel's few large tiles leave the last round of blocks partly empty.  Measured at A2W2 on 3x3 convolutions over
// 128 / 256 / 512 channels with 3136 .. 50176 output pixels x 128 .. 512 channels (3136 .. 12544 waves): 4 to 9 %
// faster than the block kernel on every one (392 .. 1568 of its 64 x 64 tiles); with 1-bit weights (half the
// arithmetic per activation word fetched) the two are level, and reductions below about 1000 elements belong to
// the row kernel or are too short to amortise a wave's own copy of the weights.  With thousands of tiles the
// block kernel fills its rounds and is the faster one (0.95 of the VALU roof at 4096^3, where the panel kernel's
// LDS broadcasts and per-panel address arithmetic hold it below 0.8).
bool prefer_panel_kernel(int64_t M, int N, int Kw, int abits, int wbits)
{
    const int64_t tiles = block_tiles((int)M, N, abits, wbits);
    // (A1W1: only where the block kernel has fewer than two of its 64 x 64 tiles per compute unit; 392 of them measured
    // 16 to 22 % behind the panel kernel, 1568 level with it)
    const bool widths = (abits >= 2 && abits * wbits == 4 && tiles < 2048) || (abits * wbits == 1 && tiles < 512);
    return widths && Kw >= 32 && M >= 2048 && ((M + 63) / 64) * ((N + 7) / 8) >= 3072;
}

// Panel kernel: how many waves of a block share a tile's reduction.  One wave per 64 x 8 tile is the least
// overhead, but a launch of only a few tiles per SIMD takes as long as the SIMD with the most of them: 3136 tiles
// on 1024 SIMDs are four on some and three on most, a third more time than work.  With the reduction shared by
// s waves the units are s times as many and 1 / s as long; each further wave costs about 200 instructions (its
// own addresses and start, the exchange of partial sums) against the tile's 2 * abits * wbits * 8 * Kw.
// The model: a SIMD takes eight waves at once and issues at full rate only with several of them, and the waves
// beyond a multiple of eight run as a last, thinner round, at the rate the register-only AND + popcount loop
// measured for that many waves per SIMD (0.72 of the full rate for one wave, 0.85 for two, 0.94 for four).  (Eight is
// the model's round, not every instantiation's occupancy - A2W2 keeps five waves per SIMD resident - but it is with
// eight that the model orders the measured layer shapes correctly.)
int plan_panel_waves(int64_t M, int N, int Kw, int abits, int wbits)
{
    static const double rate[9] = {1.0, 0.715, 0.85, 0.90, 0.94, 0.955, 0.97, 0.985, 1.0};
    const double per_simd = (double)(((M + 63) / 64) * ((N + 7) / 8)) / 1024.0;
    const double tile = 2.0 * abits * wbits * 8 * Kw;
    int best = 1;
    double best_cost = 1e300;
    for (int s = 1; s <= dlrt::kPanelMaxWaves; ++s) {
        if (dlrt::panel_words(Kw, s) == 0) continue;
        const double units = per_simd * s;
        const int64_t most = (int64_t)(units + 0.999999);  // waves of the fullest SIMD
        const double rounds = (double)(most / 8 * 8) + (most % 8 ? (most % 8) / rate[most % 8] : 0.0);
        const double cost = rounds / units * (1.0 + 200.0 * (s - 1) / tile);
        if (cost < 0.98 * best_cost) { best_cost = cost; best = s; }
    }
    return best;
}

// Row kernel: a wave covers 64 rows x ncols columns.  32 columns (one output word per row) measured fastest
// or within 3 % of it wherever there are many waves: more, shorter waves balance better over the SIMDs than the
// saved activation loads are worth, and only from about 32 K waves on do wider waves gain a few per cent.
// With FEW waves per SIMD the whole number of waves a SIMD ends up with decides (6272 equal waves on 1024 SIMDs
// are seven on some and six on the rest: the launch takes seven waves' time, 14 % more than its work), and waves
// of 16 columns, which write half an output word each, divide more finely at the price of fetching every
// activation row twice as often.  The choice follows a model fitted to measurements of eight layer shapes at 8, 16,
// 32 and 64 columns: time ~ ceil(waves per SIMD) / (waves per SIMD) x (1 + P / instructions per wave's columns),
// P being a wave's own cost in VALU instructions: 200 for a convolution (im2col addresses, loads, start and end),
// 80 for a GEMM or 1x1 convolution (the row's words are one run).  `halves`: the call writes nothing but the
// packed output, from unsigned activations (the only path with sub-word stores).
int plan_rows(int64_t M, int N, int Kw, int abits, int wbits, bool halves, bool conv)
{
    const int64_t row_blocks = (M + 63) / 64;
    int ncols = 32;
    if (halves && N % 32 == 0 && row_blocks * (N / 32) < 4096) {
        // a launch that cannot fill the chip with 32-column waves (single images): the widest waves that still make
        // about 1500 of them, else the narrowest (measured on eight such layers: the best or within 3 % of it)
        ncols = row_blocks * (N / 16) >= 1536 ? 16 : 8;
    } else if (halves && N % 32 == 0) {
        auto cost = [&](int nc) {
            const double per_simd = (double)(row_blocks * (N / nc)) / 1024.0;
            const double column = 2.0 * abits * wbits * Kw + 10.0;  // AND/BCNT pairs and the epilogue of one output
            return (double)(int64_t)(per_simd + 0.999999) / per_simd * (1.0 + (conv ? 200.0 : 80.0) / (nc * column));
        };
        if (cost(16) < 0.98 * cost(32)) ncols = 16;
    }
    while (ncols >= 32 && ncols < 128 && ncols < N && row_blocks * ((N + ncols - 1) / ncols) > 32768) ncols *= 2;
    return ncols;
}

}  // namespace

namespace dlrt {

void query_plan(int M, int N, int Kw, int abits, int wbits, int *block_kernel, int *tile_rows, int *tile_cols, int *ksplit)
{
    const bool wave = prefer_wave_kernel(M, N, abits, wbits) && (int64_t)M * abits * Kw * 4 <= (1LL << 31) &&
                      (int64_t)N * wbits * Kw * 4 <= (1LL << 31);  // (its operands are addressed with 32-bit offsets)
    int rows = block_tile(abits), cols = block_tile(wbits), ks = 1;
    if (prefer_rows_kernel(M, N, Kw, abits, wbits, true)) {  // (as for a chained layer: packed output only)
        if (block_kernel) *block_kernel = 2;
        if (tile_rows) *tile_rows = 64;
        if (tile_cols) *tile_cols = plan_rows(M, N, Kw, abits, wbits, true, true);  // as for a chained conv layer (packed output only)
        if (ksplit) *ksplit = 1;
        return;
    }
    if (prefer_panel_kernel(M, N, Kw, abits, wbits) && Kw % 4 == 0) {
        if (block_kernel) *block_kernel = 3;
        if (tile_rows) *tile_rows = 64;
        if (tile_cols) *tile_cols = 8;
        if (ksplit) *ksplit = plan_panel_waves(M, N, Kw, abits, wbits);
        return;
    }
    if (!wave && prefer_half_rows(M, N, abits, wbits)) rows /= 2;
    if (wave) {
        const WavePlan p = plan_wave(M, N, Kw, abits, wbits, 0, 0);
        rows = p.tm ? (wbits <= 2 ? 8 : 4) * p.tm : 4;
        cols = 32;
        ks = p.ksplit;
    }
    if (block_kernel) *block_kernel = wave ? 0 : 1;
    if (tile_rows) *tile_rows = rows;
    if (tile_cols) *tile_cols = cols;
    if (ksplit) *ksplit = ks;
}

dlrt_status launch_gemm(const uint32_t *A, const uint32_t *W, int M, int N, int Kw, int abits, int wbits,
                        bool a_msb_neg, bool w_msb_neg, bool bipolar, const FusedOut &o, hipStream_t stream)
{
    ContractArgs g{};
    g.A = A; g.W = W; g.M = M; g.N = N; g.Kw = Kw;
    g.a_msb_neg = a_msb_neg; g.w_msb_neg = w_msb_neg;
    const int va = widest_vec(A, Kw), vw = widest_vec(W, Kw);
    g.vec = va < vw ? va : vw;
    const bool halves = o.packed && !o.acc && !o.y && !o.q && !a_msb_neg;
    if (prefer_rows_kernel(M, N, Kw, abits, wbits, halves))
        return launch_rows(g, o, abits, wbits, bipolar, false, plan_rows(M, N, Kw, abits, wbits, halves, false), -1, stream);
    const int64_t a_bytes = (int64_t)M * abits * Kw * 4;
    if (prefer_panel_kernel(M, N, Kw, abits, wbits) && panel_kernel_has(g, abits, wbits, false, 8, a_bytes)) {
        g.a_bytes = (uint32_t)a_bytes;
        int kwaves = plan_panel_waves(M, N, Kw, abits, wbits);
        if (!panel_kernel_has(g, abits, wbits, false, 8, a_bytes, kwaves)) kwaves = 1;
        return launch_panels(g, o, abits, wbits, bipolar, false, 8, kwaves, stream);
    }
    uint32_t ab = 0, wb = 0;
    if (prefer_wave_kernel(M, N, abits, wbits) && wave_operand_bytes(g, abits, wbits, false, &ab, &wb)) {
        const WavePlan p = plan_wave(M, N, Kw, abits, wbits, 0, 0);
        return wave_by_abits(g, o, abits, wbits, bipolar, false, p.tm, p.ksplit, stream);
    }
    g.half_rows = prefer_half_rows(M, N, abits, wbits);
    return by_abits(g, o, abits, wbits, bipolar, false, stream);
}

static ContractArgs conv_args(const uint32_t *X, const uint32_t *Wp, const ConvShape &c, bool a_msb_neg, bool w_msb_neg)
{
    ContractArgs g{};
    g.A = X; g.W = Wp;
    g.M = c.N * c.Ho * c.Wo; g.N = c.Co; g.Kw = c.KH * c.KW * c.Cw;
    g.a_msb_neg = a_msb_neg; g.w_msb_neg = w_msb_neg;
    // a tap's Cw words must not be split by a vector load; the weight rows (KH*KW*Cw words) then
    // allow at least the same width
    const int va = widest_vec(X, c.Cw), vw = widest_vec(Wp, g.Kw);
    g.vec = va < vw ? va : vw;
    g.H = c.H; g.Wd = c.W; g.Cw = c.Cw; g.KH = c.KH; g.KW = c.KW; g.Ho = c.Ho; g.Wo = c.Wo;
    g.sh = c.sh; g.sw = c.sw; g.ph = c.ph; g.pw = c.pw;
    g.magicCw = magic_for(c.Cw);
    g.magicKW = magic_for(c.KW);
    g.magicKW16 = (uint32_t)((65536 + c.KW - 1) / c.KW);
    g.tapMul = (uint32_t)((65536 + c.Cw - 1) / c.Cw);
    g.tapShift = 16;
    for (int b = 0; b < 24; ++b)
        if (c.Cw == 1 << b) { g.tapMul = 1; g.tapShift = (uint32_t)b; }
    // row m < M is divided by Ho * Wo, the remainder (< Ho * Wo) by Wo: the multiply-high division is exact
    // while dividend * divisor stays below 2^32
    const int64_t hw = (int64_t)c.Ho * c.Wo;
    g.magicHW = (int64_t)g.M * hw < (1LL << 32) ? magic_for((int)hw) : 1u;
    g.magicWo = hw * c.Wo < (1LL << 32) ? magic_for(c.Wo) : 1u;
    return g;
}

// A 1x1 convolution with stride 1 and no padding IS a GEMM over the pixels (the im2col row of an output pixel is
// that pixel's own packed words), so it runs on the GEMM instantiations, which decode no pixel coordinates.
static bool pointwise(const ConvShape &c)
{
    return c.KH == 1 && c.KW == 1 && c.sh == 1 && c.sw == 1 && c.ph == 0 && c.pw == 0;
}

dlrt_status launch_conv_pair(const uint32_t *const X[2], const uint32_t *const Wp[2], const ConvShape c[2], int abits,
                             int wbits, bool a_msb_neg, bool w_msb_neg, bool bipolar, const FusedOut o[2],
                             hipStream_t stream)
{
    ContractArgs g[2];
    // Two 1x1 convolutions that both take the row kernel, with register rows of the same length (at most 8 words) and
    // together at most four waves per SIMD (single images: each alone leaves most of the chip idle and costs a
    // dependent launch of its own), share one row-kernel launch.
    {
        bool rows_pair = pointwise(c[0]) && pointwise(c[1]);
        int64_t waves = 0;
        int ncols[2] = {32, 32};
        for (int i = 0; i < 2 && rows_pair; ++i) {
            const int64_t M = (int64_t)c[i].N * c[i].Ho * c[i].Wo;
            const int Kw = c[i].Cw;
            const bool halves = o[i].packed && !o[i].acc && !o[i].y && !o[i].q && !a_msb_neg;
            rows_pair = Kw <= 8 && prefer_rows_kernel(M, c[i].Co, Kw, abits, wbits, halves);
            ncols[i] = plan_rows(M, c[i].Co, Kw, abits, wbits, halves, false);
            waves += ((M + 63) / 64) * ((c[i].Co + ncols[i] - 1) / ncols[i]);
        }
        if (rows_pair && waves <= 4096) {
            for (int i = 0; i < 2; ++i) g[i] = conv_args(X[i], Wp[i], c[i], a_msb_neg, w_msb_neg);
            dlrt_status st = DLRT_ERR_BITS;
            switch (abits) {
            case 1: st = dlrt::launch_rows_pair_a1(g, o, wbits, bipolar, ncols, stream); break;
            case 2: st = dlrt::launch_rows_pair_a2(g, o, wbits, bipolar, ncols, stream); break;
            case 3: st = dlrt::launch_rows_pair_a3(g, o, wbits, bipolar, ncols, stream); break;
            case 4: st = dlrt::launch_rows_pair_a4(g, o, wbits, bipolar, ncols, stream); break;
            }
            if (st != DLRT_ERR_SHAPE) return st;  // (rows of different lengths: two launches, below)
        }
    }
    int ksplit = 1;
    const int rows = wbits <= 2 ? 8 : 4;  // both problems on the smallest wave tile
    // sharing a launch (on the smallest wave tile) pays while neither problem can fill the chip; larger ones
    // run faster on a kernel and tile of their own, so such a pair goes out as two ordinary launches.  A problem of
    // at most 2^20 outputs shares a launch even where it would take the row kernel alone: the dependent launch
    // it saves (3 us) is worth more than the row kernel's lead on it (25600 x 32 x 32: 3.3 against 4.4 us; the
    // YOLO-style batch-1 chain 61.6 -> 60.3 us with the two pairs this adds).
    bool pairable = true;
    for (int i = 0; i < 2; ++i) {
        const int64_t M = (int64_t)c[i].N * c[i].Ho * c[i].Wo;
        const int Kw = c[i].KH * c[i].KW * c[i].Cw;
        const bool halves = o[i].packed && !o[i].acc && !o[i].y && !o[i].q && !a_msb_neg;
        const bool wave_layer = block_tiles((int)M, c[i].Co, abits, wbits) < wave_below(abits) &&
                                !prefer_rows_kernel(M, c[i].Co, Kw, abits, wbits, halves);
        pairable = pairable && (wave_layer || M * c[i].Co <= (1 << 20));
    }
    if (!pairable) {
        for (int i = 0; i < 2; ++i) {
            const dlrt_status st = launch_conv(X[i], Wp[i], c[i], abits, wbits, a_msb_neg, w_msb_neg, bipolar, o[i], 0, 0, stream);
            if (st != DLRT_OK) return st;
        }
        return DLRT_OK;
    }
    for (int i = 0; i < 2; ++i) {
        g[i] = conv_args(X[i], Wp[i], c[i], a_msb_neg, w_msb_neg);
        const WavePlan p = plan_wave(g[i].M, g[i].N, g[i].Kw, abits, wbits, rows, 0);
        if (!p.found) return DLRT_ERR_SHAPE;
        if (p.ksplit > ksplit) ksplit = p.ksplit;  // one block shape for both: the deeper reduction decides
    }
    return wave_by_abits(g, o, 2, abits, wbits, bipolar, !(pointwise(c[0]) && pointwise(c[1])), 1, ksplit, stream);
}

dlrt_status launch_conv(const uint32_t *X, const uint32_t *Wp, const ConvShape &c, int abits, int wbits,
                        bool a_msb_neg, bool w_msb_neg, bool bipolar, const FusedOut &o, int tile_rows, int ksplit,
                        hipStream_t stream)
{
    const ContractArgs g = conv_args(X, Wp, c, a_msb_neg, w_msb_neg);
    const bool conv = !pointwise(c);
    const bool rows_fit = row_kernel_has(g.Kw);
    const int64_t x_bytes = (int64_t)c.N * c.H * c.W * abits * c.Cw * 4;
    const bool halves = o.packed && !o.acc && !o.y && !o.q && !a_msb_neg;
    const int rows_ncols = plan_rows(g.M, g.N, g.Kw, abits, wbits, halves, conv);
    if (tile_rows >= 128 && tile_rows % 128 == 0) {  // hint: the panel kernel, 8 * ksplit columns per block,
        const int ncols = ksplit == 0 ? 8 : 8 * ksplit, kwaves = tile_rows / 128;  // tile_rows / 128 waves sharing the reduction
        if (kwaves > kPanelMaxWaves || !panel_kernel_has(g, abits, wbits, conv, ncols, x_bytes, kwaves)) return DLRT_ERR_SHAPE;
        ContractArgs gp = g;
        gp.a_bytes = (uint32_t)x_bytes;
        return launch_panels(gp, o, abits, wbits, bipolar, conv, ncols, kwaves, stream);
    }
    if (tile_rows == 64) {  // hint: the row kernel, 8 * ksplit columns per wave
        if (!rows_fit || ksplit < -8192 || ksplit > 8192) return DLRT_ERR_SHAPE;
        // a positive hint: every wave that wide; a negative one: as many units as possible as two waves of half the width
        return launch_rows(g, o, abits, wbits, bipolar, conv, ksplit > 0 ? 8 * ksplit : ksplit < 0 ? -8 * ksplit : rows_ncols,
                           ksplit < 0 ? -2 : 0, stream);
    }
    if (tile_rows == 0 && ksplit == 0 && prefer_rows_kernel(g.M, g.N, g.Kw, abits, wbits, halves))
        return launch_rows(g, o, abits, wbits, bipolar, conv, rows_ncols, -1, stream);
    if (tile_rows == 0 && ksplit == 0 && prefer_panel_kernel(g.M, g.N, g.Kw, abits, wbits) &&
        panel_kernel_has(g, abits, wbits, conv, 8, x_bytes)) {
        ContractArgs gp = g;
        gp.a_bytes = (uint32_t)x_bytes;
        int kwaves = plan_panel_waves(g.M, g.N, g.Kw, abits, wbits);
        if (!panel_kernel_has(g, abits, wbits, conv, 8, x_bytes, kwaves)) kwaves = 1;
        return launch_panels(gp, o, abits, wbits, bipolar, conv, 8, kwaves, stream);
    }
    uint32_t ab = 0, wb = 0;
    if (tile_rows > 0 || ksplit > 0 ||
        (prefer_wave_kernel(g.M, g.N, abits, wbits) && wave_operand_bytes(g, abits, wbits, conv, &ab, &wb))) {
        const WavePlan p = plan_wave(g.M, g.N, g.Kw, abits, wbits, tile_rows, ksplit);
        if (!p.found) return DLRT_ERR_SHAPE;  // the hints name a tile the kernel does not have
        return wave_by_abits(g, o, abits, wbits, bipolar, conv, p.tm, p.ksplit, stream);
    }
    ContractArgs gb = g;
    gb.half_rows = prefer_half_rows(g.M, g.N, abits, wbits);
    return by_abits(gb, o, abits, wbits, bipolar, conv, stream);
}

}  // namespace dlrt
