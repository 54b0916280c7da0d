/*
 * CPU oracle for ultra-low-bit GEMM / convolution (DeepliteRT, arXiv 2207.08820).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it, and
 * it shares no code, header, table or helper with the HIP sources.
 *
 * What the method computes (Section V): the bit-serial sum over bitplane pairs
 *     sum_i sum_j popcount(W[i] & A[j]) << (i + j)
 * is, exactly, the dot product of the low-bit weight and activation VALUES.
 * So the oracle is that dot product written out on the unpacked integers: it
 * never forms a bitplane in gemm/conv.  Signed operands (the quantizer of
 * Section IV emits values in [-2^(b-1), 2^(b-1)-1]) and bipolar 1-bit weights
 * are simply integer values here; how the GPU side encodes them in planes is
 * its own business.
 *
 * Values travel as int8 (range needed: -8 .. 15).  Accumulation is int32.
 * All loops are the textbook ones; OpenMP only splits the outermost loop.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Section V, multi-bit equation read as its left-hand side "W . A":
 * C[m][n] = sum_k a[m][k] * w[n][k]   (both operands K-contiguous). */
void oracle_gemm_i32(const int8_t *a, const int8_t *w, int32_t *c,
                     int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int32_t)a[m * K + k] * (int32_t)w[n * K + k];
            c[m * N + n] = s;
        }
    }
}

/* Section V applies the bit-serial dot product to convolution: a direct
 * convolution whose dot products are the integer ones above.  x: NHWC, w: OHWI,
 * y: NHWC int32.  Taps that fall outside the image are skipped, which is zero
 * padding. */
void oracle_conv2d_i32(const int8_t *x, const int8_t *w, int32_t *y,
                       int N, int H, int W, int Ci, int Co, int KH, int KW,
                       int stride_h, int stride_w, int pad_h, int pad_w)
{
    const int Ho = (H + 2 * pad_h - KH) / stride_h + 1;
    const int Wo = (W + 2 * pad_w - KW) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int oh = 0; oh < Ho; ++oh) {
            for (int ow = 0; ow < Wo; ++ow) {
                for (int co = 0; co < Co; ++co) {
                    int32_t s = 0;
                    for (int kh = 0; kh < KH; ++kh) {
                        const int ih = oh * stride_h - pad_h + kh;
                        if (ih < 0 || ih >= H) continue;
                        for (int kw = 0; kw < KW; ++kw) {
                            const int iw = ow * stride_w - pad_w + kw;
                            if (iw < 0 || iw >= W) continue;
                            const int8_t *xp = x + (((size_t)n * H + ih) * W + iw) * Ci;
                            const int8_t *wp = w + (((size_t)co * KH + kh) * KW + kw) * Ci;
                            for (int ci = 0; ci < Ci; ++ci)
                                s += (int32_t)xp[ci] * (int32_t)wp[ci];
                        }
                    }
                    y[(((size_t)n * Ho + oh) * Wo + ow) * Co + co] = s;
                }
            }
        }
    }
}

/* Section IV quantizer: t_bar = round(clip(t / s, lo, hi)), the bracket in the
 * printed formula read as round-to-nearest (ties to even, the default mode).
 * Signed: lo = -2^(b-1), hi = 2^(b-1)-1 (the Q_N, Q_P of the paper); unsigned
 * activations use lo = 0, hi = 2^b - 1.  scale: one value (per_row == 0) or one
 * per row. */
void oracle_quantize(const float *x, const float *scale, int per_row,
                     int64_t rows, int64_t K, float lo, float hi, int8_t *q)
{
    for (int64_t r = 0; r < rows; ++r) {
        const float s = scale[per_row ? r : 0];
        for (int64_t k = 0; k < K; ++k) {
            float v = x[r * K + k] / s;
            v = fminf(fmaxf(v, lo), hi);
            q[r * K + k] = (int8_t)nearbyintf(v);
        }
    }
}

/* Quantizer for bipolar (+1 / -1) one-bit weights.  Section IV with b = 1 gives
 * the range {-1, 0}, which has no +1; the bipolar encoding has no 0.  Its
 * quantizer is therefore read as the sign of t / s, zero counted as +1 (the
 * usual convention of binary networks). */
void oracle_quantize_bipolar(const float *x, const float *scale, int per_row,
                             int64_t rows, int64_t K, int8_t *q)
{
    for (int64_t r = 0; r < rows; ++r) {
        const float s = scale[per_row ? r : 0];
        for (int64_t k = 0; k < K; ++k)
            q[r * K + k] = (x[r * K + k] / s >= 0.0f) ? 1 : -1;
    }
}

/* Section IV dequantisation t_hat = t_bar * s, taken per output channel, with an
 * optional bias, as one fused multiply-add on the exactly converted integer;
 * then the quantizer of the same section (scale 1, unsigned range) for the
 * values handed to the next layer.  out_f32 / out_q may be NULL. */
void oracle_epilogue_f32(const int32_t *acc, const float *scale, const float *bias,
                         int64_t rows, int C, float *out_f32, uint8_t *out_q, int qbits)
{
    const float qmax = (float)((1 << qbits) - 1);
    for (int64_t r = 0; r < rows; ++r) {
        for (int c = 0; c < C; ++c) {
            const float y = fmaf((float)acc[r * C + c], scale[c], bias ? bias[c] : 0.0f);
            if (out_f32) out_f32[r * C + c] = y;
            if (out_q) {
                const float t = fminf(fmaxf(nearbyintf(y), 0.0f), qmax);
                out_q[r * C + c] = (uint8_t)t;
            }
        }
    }
}

/* Section V's bitplane split of weights and activations: the packed format the
 * GPU packer must emit, written out bit by bit.
 * q: rows x K values.  enc 0 = unsigned, 1 = two's complement (plane p holds bit p
 * of the b-bit pattern), 2 = bipolar (bits == 1; +1 -> bit 1, -1 -> bit 0).
 * dst: [rows][bits][ceil(K/32)] words, element k -> bit (k % 32) of word k / 32,
 * unused high bits of the last word are zero. */
void oracle_pack_bitplanes(const int8_t *q, int64_t rows, int64_t K, int bits, int enc,
                           uint32_t *dst)
{
    const int64_t Kw = (K + 31) / 32;
    memset(dst, 0, (size_t)rows * bits * Kw * sizeof(uint32_t));
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t k = 0; k < K; ++k) {
            const int v = q[r * K + k];
            unsigned pattern;
            if (enc == 2)
                pattern = v > 0 ? 1u : 0u;
            else
                pattern = (unsigned)v & ((1u << bits) - 1u);
            for (int p = 0; p < bits; ++p) {
                if ((pattern >> p) & 1u)
                    dst[(r * bits + p) * Kw + k / 32] |= 1u << (k % 32);
            }
        }
    }
}

/* Conv weights OHWI -> [Co][bits][KH*KW*Cw], Cw = ceil(Ci/32): every (kh,kw) tap
 * is padded to whole words on its own so that a tap lines up with the packed
 * NHWC activation words of one pixel. */
void oracle_pack_conv_weights(const int8_t *w, int Co, int KH, int KW, int Ci, int bits,
                              int enc, uint32_t *dst)
{
    const int Cw = (Ci + 31) / 32;
    const size_t per_co = (size_t)bits * KH * KW * Cw;
    memset(dst, 0, (size_t)Co * per_co * sizeof(uint32_t));
    for (int co = 0; co < Co; ++co) {
        for (int t = 0; t < KH * KW; ++t) {
            for (int ci = 0; ci < Ci; ++ci) {
                const int v = w[((size_t)co * KH * KW + t) * Ci + ci];
                unsigned pattern;
                if (enc == 2)
                    pattern = v > 0 ? 1u : 0u;
                else
                    pattern = (unsigned)v & ((1u << bits) - 1u);
                for (int p = 0; p < bits; ++p) {
                    if ((pattern >> p) & 1u)
                        dst[co * per_co + ((size_t)p * KH * KW + t) * Cw + ci / 32]
                            |= 1u << (ci % 32);
                }
            }
        }
    }
}
