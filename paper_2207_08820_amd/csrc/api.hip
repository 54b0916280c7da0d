// The C ABI of include/dlrt.h: argument validation on the host, then a launch.  Nothing here
// allocates, synchronises or keeps state.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlrt.h"
#include "launch.h"

namespace {

// Rows and columns are 32-bit in the kernels, which also index up to one tile (at most 128 rows or
// columns) past the end before clamping: leave that much headroom.
constexpr int64_t kMaxDim = 0x7fffffffLL - 1024;


bool bits_ok(int b) { return b >= 1 && b <= 4; }
bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }
hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

dlrt_status check_encodings(int abits, int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w)
{
    if (!bits_ok(abits) || !bits_ok(wbits)) return DLRT_ERR_BITS;
    if (enc_a != DLRT_UNSIGNED && enc_a != DLRT_TWOS) return DLRT_ERR_ENCODING;
    if (enc_w != DLRT_UNSIGNED && enc_w != DLRT_TWOS && enc_w != DLRT_BIPOLAR) return DLRT_ERR_ENCODING;
    if (enc_w == DLRT_BIPOLAR && wbits != 1) return DLRT_ERR_ENCODING;
    return DLRT_OK;
}

dlrt_status check_pack(const void *src, dlrt_src st, int bits, dlrt_encoding enc, const float *scale, const void *dst)
{
    if (!src || !dst) return DLRT_ERR_NULL;
    if (!bits_ok(bits)) return DLRT_ERR_BITS;
    if (st != DLRT_SRC_U8 && st != DLRT_SRC_I8 && st != DLRT_SRC_F32) return DLRT_ERR_SHAPE;
    if (enc != DLRT_UNSIGNED && enc != DLRT_TWOS && enc != DLRT_BIPOLAR) return DLRT_ERR_ENCODING;
    if (enc == DLRT_BIPOLAR && bits != 1) return DLRT_ERR_ENCODING;
    if (st == DLRT_SRC_F32 && !scale) return DLRT_ERR_NULL;
    if (!aligned16(dst)) return DLRT_ERR_ALIGN;
    return DLRT_OK;
}

// Validation shared by the fused convolution entry points; fills the launcher's shape and outputs.
dlrt_status check_conv_problem(const dlrt_conv_problem &p, int abits, dlrt::ConvShape &c, dlrt::FusedOut &o)
{
    if (!p.X || !p.Wp) return DLRT_ERR_NULL;
    if (!p.out_acc && !p.out_f32 && !p.out_q && !p.out_packed) return DLRT_ERR_NULL;
    if ((p.out_f32 || p.out_q || p.out_packed) && !p.scale) return DLRT_ERR_NULL;
    if ((p.out_q || p.out_packed) && !bits_ok(p.qbits)) return DLRT_ERR_BITS;
    if (p.N <= 0 || p.H <= 0 || p.W <= 0 || p.Ci <= 0 || p.Co <= 0 || p.KH <= 0 || p.KW <= 0) return DLRT_ERR_SHAPE;
    if (p.stride_h <= 0 || p.stride_w <= 0 || p.pad_h < 0 || p.pad_w < 0) return DLRT_ERR_SHAPE;
    if (p.H + 2 * p.pad_h < p.KH || p.W + 2 * p.pad_w < p.KW) return DLRT_ERR_SHAPE;
    const int Ho = (p.H + 2 * p.pad_h - p.KH) / p.stride_h + 1, Wo = (p.W + 2 * p.pad_w - p.KW) / p.stride_w + 1;
    const int64_t Cw = (p.Ci + 31) / 32;
    if ((int64_t)p.N * Ho * Wo > kMaxDim || (int64_t)p.KH * p.KW * Cw > 0x7ffffff) return DLRT_ERR_SHAPE;
    if ((int64_t)p.H * p.W * abits * Cw > 0x7fffffff) return DLRT_ERR_SHAPE;
    // the kernels divide reduction-word indices by Cw and KW with a 32-bit multiply-high
    if ((int64_t)p.KH * p.KW * Cw * (Cw > p.KW ? Cw : p.KW) > 0x7fffffff) return DLRT_ERR_SHAPE;
    if (!aligned16(p.X) || !aligned16(p.Wp) || (p.out_packed && !aligned16(p.out_packed))) return DLRT_ERR_ALIGN;
    c = dlrt::ConvShape{p.N, p.H, p.W, (int)Cw, p.Co, p.KH, p.KW, Ho, Wo, p.stride_h, p.stride_w, p.pad_h, p.pad_w};
    o = dlrt::FusedOut{};
    o.acc = p.out_acc; o.y = p.out_f32; o.q = p.out_q; o.packed = p.out_packed;
    o.scale = p.scale; o.bias = p.bias;
    o.qbits = (p.out_q || p.out_packed) ? p.qbits : 1;
    return DLRT_OK;
}

}  // namespace

extern "C" {

size_t dlrt_packed_words(int64_t rows, int64_t K, int bits)
{
    if (rows <= 0 || K <= 0 || !bits_ok(bits)) return 0;
    return (size_t)rows * (size_t)bits * (size_t)((K + 31) / 32);
}

const char *dlrt_status_string(dlrt_status status)
{
    switch (status) {
    case DLRT_OK: return "ok";
    case DLRT_ERR_NULL: return "a required pointer is NULL";
    case DLRT_ERR_BITS: return "bit width outside 1..4";
    case DLRT_ERR_SHAPE: return "non-positive or inconsistent size";
    case DLRT_ERR_ENCODING: return "encoding unknown or not allowed for this operand";
    case DLRT_ERR_ALIGN: return "packed buffer is not 16-byte aligned";
    case DLRT_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

dlrt_status dlrt_pack_bitplanes(const void *src, dlrt_src st, int64_t rows, int64_t K, int64_t ld, int bits,
                                dlrt_encoding enc, const float *scale, int scale_per_row, uint32_t *dst, void *stream)
{
    if (dlrt_status s = check_pack(src, st, bits, enc, scale, dst)) return s;
    if (rows <= 0 || K <= 0 || ld < K) return DLRT_ERR_SHAPE;
    const int64_t Kw = (K + 31) / 32;
    if (rows > 0x7fffffffLL * 32 / Kw) return DLRT_ERR_SHAPE;
    dlrt::PackArgs p{};
    p.src = src; p.src_type = st; p.rows = rows; p.K = K; p.ld = ld; p.bits = bits; p.enc = enc;
    p.scale = scale; p.scale_per_row = scale_per_row != 0; p.dst = dst;
    p.taps = 1; p.outer_stride = bits * Kw; p.plane_stride = Kw; p.tap_stride = 0;
    return dlrt::launch_pack(p, as_stream(stream));
}

namespace {

dlrt_status pack_conv_weights(const void *w_ohwi, dlrt_src st, int Co, int KH, int KW, int Ci, int bits,
                              dlrt_encoding enc, const float *scale, int scale_per_channel, uint32_t *dst, void *stream)
{
    if (dlrt_status s = check_pack(w_ohwi, st, bits, enc, scale, dst)) return s;
    if (Co <= 0 || KH <= 0 || KW <= 0 || Ci <= 0) return DLRT_ERR_SHAPE;
    const int64_t Cw = (Ci + 31) / 32, taps = (int64_t)KH * KW;
    if ((int64_t)Co * taps > 0x7fffffffLL * 32 / Cw) return DLRT_ERR_SHAPE;
    dlrt::PackArgs p{};
    p.src = w_ohwi; p.src_type = st; p.rows = (int64_t)Co * taps; p.K = Ci; p.ld = Ci; p.bits = bits; p.enc = enc;
    p.scale = scale; p.scale_per_row = scale_per_channel ? 2 : 0; p.dst = dst;
    p.taps = taps; p.outer_stride = bits * taps * Cw; p.plane_stride = taps * Cw; p.tap_stride = Cw;
    return dlrt::launch_pack(p, as_stream(stream));
}

}  // namespace

dlrt_status dlrt_pack_conv_weights(const void *w_ohwi, dlrt_src st, int Co, int KH, int KW, int Ci, int bits,
                                   dlrt_encoding enc, const float *scale, uint32_t *dst, void *stream)
{
    return pack_conv_weights(w_ohwi, st, Co, KH, KW, Ci, bits, enc, scale, 0, dst, stream);
}

dlrt_status dlrt_pack_conv_weights_per_channel(const void *w_ohwi, dlrt_src st, int Co, int KH, int KW, int Ci, int bits,
                                               dlrt_encoding enc, const float *scale, uint32_t *dst, void *stream)
{
    if (st == DLRT_SRC_F32 && !scale) return DLRT_ERR_NULL;
    return pack_conv_weights(w_ohwi, st, Co, KH, KW, Ci, bits, enc, scale, 1, dst, stream);
}

dlrt_status dlrt_bitserial_gemm(const uint32_t *A, const uint32_t *W, int32_t *C, int64_t M, int64_t N, int64_t K,
                                int abits, int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w, void *stream)
{
    if (!A || !W || !C) return DLRT_ERR_NULL;
    if (dlrt_status s = check_encodings(abits, wbits, enc_a, enc_w)) return s;
    if (M <= 0 || N <= 0 || K <= 0) return DLRT_ERR_SHAPE;
    const int64_t Kw = (K + 31) / 32;
    if (M > kMaxDim || N > kMaxDim || Kw > 0x7ffffff) return DLRT_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(W)) return DLRT_ERR_ALIGN;
    dlrt::FusedOut o{};
    o.acc = C;
    o.qbits = 1;
    return dlrt::launch_gemm(A, W, (int)M, (int)N, (int)Kw, abits, wbits, enc_a == DLRT_TWOS, enc_w == DLRT_TWOS,
                             enc_w == DLRT_BIPOLAR, o, as_stream(stream));
}

dlrt_status dlrt_bitserial_gemm_fused(const uint32_t *A, const uint32_t *W, const float *scale, const float *bias, int64_t M,
                                      int64_t N, int64_t K, int abits, int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w,
                                      int32_t *out_acc, float *out_f32, uint8_t *out_q, uint32_t *out_packed, int qbits,
                                      void *stream)
{
    if (!A || !W) return DLRT_ERR_NULL;
    if (!out_acc && !out_f32 && !out_q && !out_packed) return DLRT_ERR_NULL;
    if ((out_f32 || out_q || out_packed) && !scale) return DLRT_ERR_NULL;
    if (dlrt_status s = check_encodings(abits, wbits, enc_a, enc_w)) return s;
    if ((out_q || out_packed) && !bits_ok(qbits)) return DLRT_ERR_BITS;
    if (M <= 0 || N <= 0 || K <= 0) return DLRT_ERR_SHAPE;
    const int64_t Kw = (K + 31) / 32;
    if (M > kMaxDim || N > kMaxDim || Kw > 0x7ffffff) return DLRT_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(W) || (out_packed && !aligned16(out_packed))) return DLRT_ERR_ALIGN;
    dlrt::FusedOut o{};
    o.acc = out_acc; o.y = out_f32; o.q = out_q; o.packed = out_packed;
    o.scale = scale; o.bias = bias;
    o.qbits = (out_q || out_packed) ? qbits : 1;
    return dlrt::launch_gemm(A, W, (int)M, (int)N, (int)Kw, abits, wbits, enc_a == DLRT_TWOS, enc_w == DLRT_TWOS,
                             enc_w == DLRT_BIPOLAR, o, as_stream(stream));
}

dlrt_status dlrt_bitserial_conv2d(const uint32_t *X, const uint32_t *Wp, int32_t *Y, int N, int H, int W, int Ci,
                                  int Co, int KH, int KW, int stride_h, int stride_w, int pad_h, int pad_w, int abits,
                                  int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w, void *stream)
{
    if (!X || !Wp || !Y) return DLRT_ERR_NULL;
    if (dlrt_status s = check_encodings(abits, wbits, enc_a, enc_w)) return s;
    if (N <= 0 || H <= 0 || W <= 0 || Ci <= 0 || Co <= 0 || KH <= 0 || KW <= 0) return DLRT_ERR_SHAPE;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return DLRT_ERR_SHAPE;
    if (H + 2 * pad_h < KH || W + 2 * pad_w < KW) return DLRT_ERR_SHAPE;
    const int Ho = (H + 2 * pad_h - KH) / stride_h + 1, Wo = (W + 2 * pad_w - KW) / stride_w + 1;
    const int64_t Cw = (Ci + 31) / 32;
    if ((int64_t)N * Ho * Wo > kMaxDim || (int64_t)KH * KW * Cw > 0x7ffffff) return DLRT_ERR_SHAPE;
    if ((int64_t)H * W * abits * Cw > 0x7fffffff) return DLRT_ERR_SHAPE;
    // the kernels divide reduction-word indices by Cw and KW with a 32-bit multiply-high
    if ((int64_t)KH * KW * Cw * (Cw > KW ? Cw : KW) > 0x7fffffff) return DLRT_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Wp)) return DLRT_ERR_ALIGN;
    dlrt::ConvShape c{N, H, W, (int)Cw, Co, KH, KW, Ho, Wo, stride_h, stride_w, pad_h, pad_w};
    dlrt::FusedOut o{};
    o.acc = Y;
    o.qbits = 1;
    return dlrt::launch_conv(X, Wp, c, abits, wbits, enc_a == DLRT_TWOS, enc_w == DLRT_TWOS, enc_w == DLRT_BIPOLAR, o, 0, 0,
                             as_stream(stream));
}

dlrt_status dlrt_bitserial_conv2d_fused(const uint32_t *X, const uint32_t *Wp, const float *scale, const float *bias,
                                        int N, int H, int W, int Ci, int Co, int KH, int KW, int stride_h,
                                        int stride_w, int pad_h, int pad_w, int abits, int wbits, dlrt_encoding enc_a,
                                        dlrt_encoding enc_w, int32_t *out_acc, float *out_f32, uint8_t *out_q,
                                        uint32_t *out_packed, int qbits, int tile_rows, int ksplit, void *stream)
{
    if (dlrt_status s = check_encodings(abits, wbits, enc_a, enc_w)) return s;
    if (tile_rows < 0 || (ksplit < 0 && tile_rows != 64)) return DLRT_ERR_SHAPE;  // (a negative width is a row-kernel hint)
    const dlrt_conv_problem p{X, Wp, scale, bias, N, H, W, Ci, Co, KH, KW, stride_h, stride_w, pad_h, pad_w,
                              out_acc, out_f32, out_q, out_packed, qbits};
    dlrt::ConvShape c{};
    dlrt::FusedOut o{};
    if (dlrt_status s = check_conv_problem(p, abits, c, o)) return s;
    return dlrt::launch_conv(X, Wp, c, abits, wbits, enc_a == DLRT_TWOS, enc_w == DLRT_TWOS, enc_w == DLRT_BIPOLAR, o,
                             tile_rows, ksplit, as_stream(stream));
}

dlrt_status dlrt_bitserial_conv2d_fused_pair(const dlrt_conv_problem *first, const dlrt_conv_problem *second, int abits,
                                             int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w, void *stream)
{
    if (!first || !second) return DLRT_ERR_NULL;
    if (dlrt_status s = check_encodings(abits, wbits, enc_a, enc_w)) return s;
    dlrt::ConvShape c[2];
    dlrt::FusedOut o[2];
    if (dlrt_status s = check_conv_problem(*first, abits, c[0], o[0])) return s;
    if (dlrt_status s = check_conv_problem(*second, abits, c[1], o[1])) return s;
    const uint32_t *X[2] = {first->X, second->X}, *Wp[2] = {first->Wp, second->Wp};
    return dlrt::launch_conv_pair(X, Wp, c, abits, wbits, enc_a == DLRT_TWOS, enc_w == DLRT_TWOS, enc_w == DLRT_BIPOLAR,
                                  o, as_stream(stream));
}

dlrt_status dlrt_query_plan(int64_t M, int64_t N, int64_t K, int abits, int wbits, int *block_kernel, int *tile_rows,
                            int *tile_cols, int *ksplit)
{
    if (!bits_ok(abits) || !bits_ok(wbits)) return DLRT_ERR_BITS;
    if (M <= 0 || N <= 0 || K <= 0) return DLRT_ERR_SHAPE;
    const int64_t Kw = (K + 31) / 32;
    if (M > kMaxDim || N > kMaxDim || Kw > 0x7ffffff) return DLRT_ERR_SHAPE;
    dlrt::query_plan((int)M, (int)N, (int)Kw, abits, wbits, block_kernel, tile_rows, tile_cols, ksplit);
    return DLRT_OK;
}

dlrt_status dlrt_unpacked_gemm_i8(const int8_t *A, const int8_t *W, int32_t *C, int64_t M, int64_t N, int64_t K,
                                  void *stream)
{
    if (!A || !W || !C) return DLRT_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || K % 16 != 0) return DLRT_ERR_SHAPE;
    if (M > kMaxDim || N > kMaxDim || K > 0x7fffffff) return DLRT_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(W)) return DLRT_ERR_ALIGN;
    return dlrt::launch_unpacked_gemm_i8(A, W, C, (int)M, (int)N, (int)K, as_stream(stream));
}

dlrt_status dlrt_pack_nibbles(const int8_t *src, int64_t rows, int64_t K, uint32_t *dst, void *stream)
{
    if (!src || !dst) return DLRT_ERR_NULL;
    if (rows <= 0 || K <= 0 || K % 32 != 0) return DLRT_ERR_SHAPE;
    if (rows > kMaxDim || K > 0x7fffffff) return DLRT_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return DLRT_ERR_ALIGN;
    return dlrt::launch_pack_nibbles(src, rows, K, dst, as_stream(stream));
}

dlrt_status dlrt_unpacked_gemm_i4(const uint32_t *A, const uint32_t *W, int32_t *C, int64_t M, int64_t N, int64_t K,
                                  void *stream)
{
    if (!A || !W || !C) return DLRT_ERR_NULL;
    if (M <= 0 || N <= 0 || K <= 0 || K % 32 != 0) return DLRT_ERR_SHAPE;
    if (M > kMaxDim || N > kMaxDim || K > 0x7fffffff) return DLRT_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(W)) return DLRT_ERR_ALIGN;
    return dlrt::launch_unpacked_gemm_i4(A, W, C, (int)M, (int)N, (int)K, as_stream(stream));
}

dlrt_status dlrt_epilogue_f32(const int32_t *acc, const float *scale, const float *bias, int64_t rows, int C,
                              float *out_f32, uint8_t *out_q, int qbits, void *stream)
{
    if (!acc || !scale || (!out_f32 && !out_q)) return DLRT_ERR_NULL;
    if (rows <= 0 || C <= 0) return DLRT_ERR_SHAPE;
    if (out_q && (qbits < 1 || qbits > 8)) return DLRT_ERR_BITS;
    return dlrt::launch_epilogue(acc, scale, bias, rows, C, out_f32, out_q, out_q ? qbits : 1, as_stream(stream));
}

}  // extern "C"
