// Host-side set-up of a contraction launch: operand alignment, convolution geometry, and the
// choice of the per-bit-width translation unit of contract.hip.
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

dlrt_status by_abits(const dlrt::ContractArgs &g, int abits, int wbits, bool bipolar, bool conv, hipStream_t stream)
{
    switch (abits) {
    case 1: return dlrt::launch_contract_a1(g, wbits, bipolar, conv, stream);
    case 2: return dlrt::launch_contract_a2(g, wbits, bipolar, conv, stream);
    case 3: return dlrt::launch_contract_a3(g, wbits, bipolar, conv, stream);
    case 4: return dlrt::launch_contract_a4(g, wbits, bipolar, conv, stream);
    }
    return DLRT_ERR_BITS;
}

}  // namespace

namespace dlrt {

dlrt_status launch_gemm(const uint32_t *A, const uint32_t *W, int32_t *C, int M, int N, int Kw, int abits,
                        int wbits, bool a_msb_neg, bool w_msb_neg, bool bipolar, hipStream_t stream)
{
    ContractArgs g{};
    g.A = A; g.W = W; g.C = C; g.M = M; g.N = N; g.Kw = Kw;
    g.a_msb_neg = a_msb_neg; g.w_msb_neg = w_msb_neg;
    const int va = widest_vec(A, Kw), vw = widest_vec(W, Kw);
    g.vec = va < vw ? va : vw;
    return by_abits(g, abits, wbits, bipolar, false, stream);
}

dlrt_status launch_conv(const uint32_t *X, const uint32_t *Wp, int32_t *Y, int N, int H, int W, int Cw, int Co,
                        int KH, int KW, int Ho, int Wo, int sh, int sw, int ph, int pw, int abits, int wbits,
                        bool a_msb_neg, bool w_msb_neg, bool bipolar, hipStream_t stream)
{
    ContractArgs g{};
    g.A = X; g.W = Wp; g.C = Y;
    g.M = N * Ho * Wo; g.N = Co; g.Kw = KH * KW * Cw;
    g.a_msb_neg = a_msb_neg; g.w_msb_neg = w_msb_neg;
    // a tap's Cw words must not be split by a vector load; the weight rows (KH*KW*Cw words) then
    // allow at least the same width
    const int va = widest_vec(X, Cw), vw = widest_vec(Wp, g.Kw);
    g.vec = va < vw ? va : vw;
    g.H = H; g.Wd = W; g.Cw = Cw; g.KH = KH; g.KW = KW; g.Ho = Ho; g.Wo = Wo;
    g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw;
    g.magicCw = magic_for(Cw);
    g.magicKW = magic_for(KW);
    return by_abits(g, abits, wbits, bipolar, true, stream);
}

}  // namespace dlrt
