/*
 * Host-only driver for tests/test_oracle_sanitized.py: calls every function of oracle/dlrt_oracle.c on
 * exactly-sized heap buffers over a spread of small and ragged shapes, so that AddressSanitizer /
 * UndefinedBehaviorSanitizer (the file is compiled with both) report any access outside a buffer, any
 * misaligned or overflowing operation.  Values are a fixed linear congruential sequence; results are not
 * checked here (the pins do that), only folded into a checksum so that nothing is optimised away.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_gemm_i32(const int8_t *a, const int8_t *w, int32_t *c, int64_t M, int64_t N, int64_t K);
void oracle_conv2d_i32(const int8_t *x, const int8_t *w, int32_t *y, int N, int H, int W, int Ci, int Co, int KH, int KW,
                       int stride_h, int stride_w, int pad_h, int pad_w);
void oracle_quantize(const float *x, const float *scale, int per_row, int64_t rows, int64_t K, float lo, float hi, int8_t *q);
void oracle_epilogue_f32(const int32_t *acc, const float *scale, const float *bias, int64_t rows, int C, float *out_f32,
                         uint8_t *out_q, int qbits);
void oracle_pack_bitplanes(const int8_t *q, int64_t rows, int64_t K, int bits, int enc, uint32_t *dst);
void oracle_pack_conv_weights(const int8_t *w, int Co, int KH, int KW, int Ci, int bits, int enc, uint32_t *dst);

static uint32_t state = 2207u;
static int next_value(int lo, int hi)
{
    state = state * 1664525u + 1013904223u;
    return lo + (int)((state >> 8) % (uint32_t)(hi - lo + 1));
}

static int8_t *values(size_t n, int lo, int hi)
{
    int8_t *p = malloc(n ? n : 1);
    for (size_t i = 0; i < n; ++i) p[i] = (int8_t)next_value(lo, hi);
    return p;
}

int main(void)
{
    uint64_t sum = 0;
    static const int sizes[] = {1, 2, 31, 32, 33, 64, 65, 100};
    const int ns = (int)(sizeof sizes / sizeof sizes[0]);
    for (int bits = 1; bits <= 4; ++bits) {
        for (int enc = 0; enc <= 2; ++enc) {
            if (enc == 2 && bits != 1) continue;
            const int lo = enc == 0 ? 0 : enc == 1 ? -(1 << (bits - 1)) : -1;
            const int hi = enc == 0 ? (1 << bits) - 1 : enc == 1 ? (1 << (bits - 1)) - 1 : 1;
            for (int i = 0; i < ns; ++i) {
                const int64_t rows = sizes[(i * 3 + bits) % ns], K = sizes[i];
                int8_t *q = values((size_t)(rows * K), lo, hi);
                if (enc == 2)
                    for (int64_t t = 0; t < rows * K; ++t) q[t] = q[t] > 0 ? 1 : -1;
                const int64_t Kw = (K + 31) / 32;
                uint32_t *dst = malloc((size_t)(rows * bits * Kw) * sizeof(uint32_t));
                oracle_pack_bitplanes(q, rows, K, bits, enc, dst);
                for (int64_t t = 0; t < rows * bits * Kw; ++t) sum += dst[t];
                free(dst);
                /* the same values as a [Co][KH][KW][Ci] weight tensor, for a few tap shapes */
                for (int kh = 1; kh <= 3; kh += 2) {
                    const int kw = kh == 1 ? 1 : 2, Ci = (int)K, Co = 3;
                    int8_t *w = values((size_t)Co * kh * kw * Ci, lo, hi);
                    const size_t words = (size_t)Co * bits * kh * kw * ((Ci + 31) / 32);
                    uint32_t *wd = malloc(words * sizeof(uint32_t));
                    oracle_pack_conv_weights(w, Co, kh, kw, Ci, bits, enc, wd);
                    for (size_t t = 0; t < words; ++t) sum += wd[t];
                    free(wd);
                    free(w);
                }
                free(q);
            }
        }
    }
    for (int i = 0; i < ns; ++i)
        for (int j = 0; j < ns; j += 2) {
            const int64_t M = sizes[i], N = sizes[j], K = sizes[(i + j) % ns];
            int8_t *a = values((size_t)(M * K), 0, 15), *w = values((size_t)(N * K), -8, 7);
            int32_t *c = malloc((size_t)(M * N) * sizeof(int32_t));
            oracle_gemm_i32(a, w, c, M, N, K);
            float *scale = malloc((size_t)N * sizeof(float)), *bias = malloc((size_t)N * sizeof(float));
            for (int64_t n = 0; n < N; ++n) {
                scale[n] = 0.001f * (float)next_value(1, 50);
                bias[n] = 0.25f * (float)next_value(-8, 8);
            }
            float *y = malloc((size_t)(M * N) * sizeof(float));
            uint8_t *qq = malloc((size_t)(M * N));
            oracle_epilogue_f32(c, scale, j % 4 ? bias : NULL, M, (int)N, y, qq, 1 + (i % 4));
            oracle_epilogue_f32(c, scale, bias, M, (int)N, NULL, qq, 4);
            oracle_epilogue_f32(c, scale, NULL, M, (int)N, y, NULL, 2);
            for (int64_t t = 0; t < M * N; ++t) sum += (uint64_t)(uint32_t)c[t] + qq[t];
            /* quantizer on the fp32 result: one scale, then one per row */
            int8_t *q8 = malloc((size_t)(M * N));
            float *rs = malloc((size_t)M * sizeof(float));
            for (int64_t m = 0; m < M; ++m) rs[m] = 0.5f + 0.125f * (float)next_value(0, 16);
            oracle_quantize(y, rs, 0, M, N, -8.0f, 7.0f, q8);
            oracle_quantize(y, rs, 1, M, N, 0.0f, 3.0f, q8);
            for (int64_t t = 0; t < M * N; ++t) sum += (uint8_t)q8[t];
            free(rs); free(q8); free(qq); free(y); free(bias); free(scale); free(c); free(w); free(a);
        }
    static const int conv[][9] = {/* N, H, W, Ci, Co, KH, KW, stride, pad */
        {1, 5, 5, 3, 2, 3, 3, 1, 1}, {2, 7, 4, 33, 5, 3, 3, 2, 1}, {1, 1, 1, 64, 1, 1, 1, 1, 0}, {1, 6, 9, 8, 3, 5, 3, 1, 2},
        {3, 4, 4, 1, 1, 1, 1, 2, 0}, {1, 8, 8, 32, 4, 2, 2, 2, 0}, {1, 3, 3, 4, 2, 3, 3, 1, 3}, {1, 9, 2, 5, 2, 1, 2, 3, 1}};
    for (size_t t = 0; t < sizeof conv / sizeof conv[0]; ++t) {
        const int *p = conv[t];
        const int N = p[0], H = p[1], W = p[2], Ci = p[3], Co = p[4], KH = p[5], KW = p[6], s = p[7], pad = p[8];
        const int Ho = (H + 2 * pad - KH) / s + 1, Wo = (W + 2 * pad - KW) / s + 1;
        if (Ho <= 0 || Wo <= 0) continue;
        int8_t *x = values((size_t)N * H * W * Ci, 0, 3), *w = values((size_t)Co * KH * KW * Ci, -2, 1);
        int32_t *y = malloc((size_t)N * Ho * Wo * Co * sizeof(int32_t));
        oracle_conv2d_i32(x, w, y, N, H, W, Ci, Co, KH, KW, s, s, pad, pad);
        for (size_t i = 0; i < (size_t)N * Ho * Wo * Co; ++i) sum += (uint32_t)y[i];
        free(y); free(w); free(x);
    }
    printf("checksum %llu\n", (unsigned long long)sum);
    return 0;
}
