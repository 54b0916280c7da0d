/*
 * dlrt.h - C ABI of the MI355X (gfx950) bit-serial low-bit GEMM / convolution library.
 *
 * The operations are those of DeepliteRT (arXiv 2207.08820): operands quantized to 1-4 bits
 * (Section IV) are split into bitplanes (Section V), every dot product is
 *      sum_i sum_j  s_w(i) s_a(j) 2^(i+j) popcount(W[i] & A[j])          (Section V, multi-bit equation)
 * accumulated in int32, and the result is dequantized by a scale (Section IV, t_hat = t_bar * s).
 *
 * Conventions shared by every call
 *   - Every pointer is a DEVICE pointer owned by the caller, except where a parameter says "host".
 *   - The library allocates nothing, keeps no state between calls and never synchronises:
 *     each call validates its arguments on the host, enqueues its kernels on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and returns.
 *   - Buffers must stay alive until the stream has passed the call.  Output buffers are fully
 *     overwritten; inputs are never written.
 *   - Argument errors return a specific DLRT_ERR_* code and enqueue nothing.  A failed launch
 *     returns DLRT_ERR_LAUNCH.
 *   - Packed operand format ("bitplane tensor"): uint32 words, [rows][bits][Kw], Kw = ceil(K/32).
 *     Element k of a row occupies bit (k % 32) of word (k / 32) of each plane; plane p holds bit p
 *     of the element's pattern (plane 0 = least significant).  Bits beyond K are zero.
 *     Packed buffers must be 16-byte aligned (DLRT_ERR_ALIGN otherwise).
 *   - Overflow is a precondition, not checked: K_total * max|a| * max|w| < 2^31, where the largest
 *     magnitude of a b-bit operand is 2^b - 1 (unsigned), 2^(b-1) (two's complement) or 1 (bipolar),
 *     and K_total is the reduction length (KH * KW * Ci for a convolution).
 */
#ifndef DLRT_H
#define DLRT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DLRT_OK = 0,
    DLRT_ERR_NULL = 1,     /* a required pointer is NULL                               */
    DLRT_ERR_BITS = 2,     /* a bit width outside 1..4                                 */
    DLRT_ERR_SHAPE = 3,    /* a non-positive or inconsistent size                      */
    DLRT_ERR_ENCODING = 4, /* unknown encoding, or one not allowed for that operand    */
    DLRT_ERR_ALIGN = 5,    /* a packed buffer is not 16-byte aligned                   */
    DLRT_ERR_LAUNCH = 6    /* the HIP runtime refused the launch                       */
} dlrt_status;

/* How a b-bit pattern maps to a value.  Section V states the unipolar {0,1} planes; the signed
 * ranges are the quantizer's of Section IV. */
typedef enum {
    DLRT_UNSIGNED = 0, /* value = sum_p 2^p bit_p                      in [0, 2^b - 1]            */
    DLRT_TWOS = 1,     /* as above but plane b-1 weighs -2^(b-1)       in [-2^(b-1), 2^(b-1) - 1] */
    DLRT_BIPOLAR = 2   /* b must be 1: bit 1 -> +1, bit 0 -> -1 (weights only)                    */
} dlrt_encoding;

typedef enum {
    DLRT_SRC_U8 = 0, /* uint8 holding the value (unsigned) or its low bits                  */
    DLRT_SRC_I8 = 1, /* int8 holding the value                                              */
    DLRT_SRC_F32 = 2 /* float32, quantized on the fly: q = round(clip(x / s, lo, hi))       */
} dlrt_src;

/* Number of uint32 words of a packed [rows][bits][ceil(K/32)] tensor; 0 if an argument is invalid. */
size_t dlrt_packed_words(int64_t rows, int64_t K, int bits);

/* Static, NUL-terminated description of a status code (host memory, never freed). */
const char *dlrt_status_string(dlrt_status status);

/*
 * Bitplane split (Section V) with the optional forward quantizer of Section IV in front.
 *   src    rows x K elements of type `st`, element (r, k) at src[r * ld + k]; ld >= K.
 *   scale  NULL, or for DLRT_SRC_F32 (required there): one float (scale_per_row == 0) or `rows`
 *          floats, all positive.  q = rint(min(max(x / s, lo), hi)), ties to even, [lo, hi] the range of
 *          `enc`.  DLRT_BIPOLAR has no zero level: there q is the sign of x / s with zero counted as +1
 *          (bit = x / s >= 0), the quantizer of binary networks.
 *          Integer sources are taken as already quantized: the low `bits` bits of the two's
 *          complement pattern are packed (bipolar: bit = value > 0); `scale` is ignored.
 *   dst    [rows][bits][ceil(K/32)] words, fully written.
 * For NHWC activations call with rows = N*H*W, K = C.
 */
dlrt_status dlrt_pack_bitplanes(const void *src, dlrt_src st, int64_t rows, int64_t K, int64_t ld,
                                int bits, dlrt_encoding enc, const float *scale, int scale_per_row,
                                uint32_t *dst, void *stream);

/*
 * Convolution weights, OHWI [Co][KH][KW][Ci] -> [Co][bits][KH*KW*Cw] words, Cw = ceil(Ci/32): every
 * (kh, kw) tap is padded to whole words on its own, so that tap t of plane p starts at word
 * (p*KH*KW + t) * Cw of its output channel and lines up with one pixel's packed NHWC words.
 * scale: as above but one float for the whole tensor (F32 source only).
 */
dlrt_status dlrt_pack_conv_weights(const void *w_ohwi, dlrt_src st, int Co, int KH, int KW, int Ci,
                                   int bits, dlrt_encoding enc, const float *scale, uint32_t *dst,
                                   void *stream);

/*
 * The same with Section IV's scale s taken per OUTPUT CHANNEL: scale holds Co floats and element
 * (co, kh, kw, ci) is quantized with scale[co] (F32 source; ignored for integer sources, may then be NULL).
 * Everything else as dlrt_pack_conv_weights.
 */
dlrt_status dlrt_pack_conv_weights_per_channel(const void *w_ohwi, dlrt_src st, int Co, int KH, int KW,
                                               int Ci, int bits, dlrt_encoding enc, const float *scale,
                                               uint32_t *dst, void *stream);

/*
 * Bit-serial GEMM (Section V, multi-bit equation applied to every (m, n) pair):
 *   C[m][n] = sum_k a[m][k] * w[n][k]      int32, row-major, leading dimension N.
 *   A  packed [M][abits][Kw], W packed [N][wbits][Kw]; both reduce along their packed axis.
 *   enc_a: UNSIGNED or TWOS.  enc_w: UNSIGNED, TWOS, or BIPOLAR (then wbits must be 1 and
 *   C = sum_j s_a(j) 2^j (2 popcount(A[j] & W) - popcount(A[j]))).
 */
dlrt_status dlrt_bitserial_gemm(const uint32_t *A, const uint32_t *W, int32_t *C,
                                int64_t M, int64_t N, int64_t K, int abits, int wbits,
                                dlrt_encoding enc_a, dlrt_encoding enc_w, void *stream);

/*
 * dlrt_bitserial_gemm with the epilogue of Section IV fused in (one launch, the int32 tensor need not
 * be written):  acc = the int32 result above;  y = fmaf((float)acc, scale[n], bias ? bias[n] : 0.0f);
 * q = (uint8) min(max(rint(y), 0), 2^qbits - 1);  out_packed = bitplanes of q, [M][qbits][ceil(N/32)]
 * words (what dlrt_pack_bitplanes would make of q).  Any of the four outputs may be NULL, not all;
 * scale [N] is required unless only out_acc is given; bias [N] may be NULL; qbits in 1..4 is read when
 * out_q or out_packed is given; out_packed must be 16-byte aligned.
 */
dlrt_status dlrt_bitserial_gemm_fused(const uint32_t *A, const uint32_t *W, const float *scale,
                                      const float *bias, int64_t M, int64_t N, int64_t K, int abits,
                                      int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w, int32_t *out_acc,
                                      float *out_f32, uint8_t *out_q, uint32_t *out_packed, int qbits,
                                      void *stream);

/*
 * Bit-serial convolution (Section V: the convolution's dot products computed bit-serially), as an
 * implicit im2col over packed NHWC activations; zero padding (an out-of-image tap contributes 0,
 * also for bipolar weights).
 *   X   packed [N][H][W][abits][Cw]   (dlrt_pack_bitplanes with rows = N*H*W, K = Ci)
 *   Wp  packed [Co][wbits][KH*KW*Cw]  (dlrt_pack_conv_weights)
 *   Y   int32 NHWC [N][Ho][Wo][Co],  Ho = (H + 2*pad_h - KH) / stride_h + 1, same for Wo.
 */
dlrt_status dlrt_bitserial_conv2d(const uint32_t *X, const uint32_t *Wp, int32_t *Y,
                                  int N, int H, int W, int Ci, int Co, int KH, int KW,
                                  int stride_h, int stride_w, int pad_h, int pad_w,
                                  int abits, int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w,
                                  void *stream);

/*
 * Convolution with the epilogue fused in, for chained layers (Section V's convolution followed by
 * Section IV's t_hat = t_bar * s and the quantizer for the next layer), as ONE launch:
 *   acc = the int32 result of dlrt_bitserial_conv2d on the same X, Wp and geometry
 *   y   = fmaf((float)acc, scale[co], bias ? bias[co] : 0.0f)
 *   q   = (uint8) min(max(rint(y), 0), 2^qbits - 1)
 *   out_packed = bitplanes of q, [N*Ho*Wo][qbits][ceil(Co/32)] words: exactly what
 *                dlrt_pack_bitplanes(q, DLRT_SRC_U8, rows = N*Ho*Wo, K = Co, qbits, DLRT_UNSIGNED)
 *                would write, i.e. the next layer's X.
 * Any of out_acc, out_f32, out_q, out_packed may be NULL, not all of them; scale is required unless
 * only out_acc is given; bias may be NULL; qbits in 1..4 (read when out_q or out_packed is given).
 * out_packed must be 16-byte aligned.  tile_rows and ksplit are tuning hints for the latency-oriented
 * kernel that small layers get: 0 lets the library plan (large problems then take the throughput kernel,
 * which has no hints); otherwise tile_rows is the number of output pixels per wave tile (4, 8, 16 or 32 for
 * wbits <= 2; 4, 8 or 16 for wbits >= 3) and ksplit (1, 2, 4, 8) the number of waves that split the
 * reduction; a combination the kernels do not have (more than 72 accumulators per lane, or more
 * than 64 KB of LDS per block) returns DLRT_ERR_SHAPE.  tile_rows = 64 asks for the row kernel (one output
 * pixel per lane; convolutions with KH*KW*ceil(Ci/32) <= 16 or = 18, DLRT_ERR_SHAPE otherwise);
 * ksplit then is the number of 8-column groups a wave covers (0: planned; 4 n for whole output words, or 1 or 2,
 * which need Co a multiple of 32, unsigned activations and no output but out_packed; DLRT_ERR_SHAPE
 * otherwise; a negative count -n: units of 8 n columns of which as many as the chip's dies all have go out as
 * two waves of 4 n columns each, the form the planner gives the last units of a large launch; 4 n must
 * itself be a width that exists).  tile_rows = 128 asks for the panel
 * kernel (one output pixel per lane, the reduction walked in panels against weights held in LDS; needs Ci a
 * multiple of 128, abits * wbits * 8 * ksplit <= 64 and at most 2^31 bytes of activations, DLRT_ERR_SHAPE
 * otherwise); ksplit (0 or 1, 2, 4) then is the number of 8-column groups a wave covers.  The result does not
 * depend on the hints.
 */
dlrt_status dlrt_bitserial_conv2d_fused(const uint32_t *X, const uint32_t *Wp, const float *scale,
                                        const float *bias, int N, int H, int W, int Ci, int Co, int KH,
                                        int KW, int stride_h, int stride_w, int pad_h, int pad_w,
                                        int abits, int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w,
                                        int32_t *out_acc, float *out_f32, uint8_t *out_q,
                                        uint32_t *out_packed, int qbits, int tile_rows, int ksplit,
                                        void *stream);

/*
 * Two fused convolutions in ONE launch: layers that do not depend on each other (typically two that read
 * the same activations, like a stride-2 3x3 conv and the 1x1 downsample conv beside it) share the fixed
 * cost of a launch, which dominates batch-1 layers.  Each problem computes exactly what
 * dlrt_bitserial_conv2d_fused computes for the same fields; both use the latency-oriented kernel with its
 * smallest tile, or, two 1x1 stride-1 convolutions over at most 256 channels each that both take the row kernel
 * and whose reductions fill register rows of the same length (1, 2, 4 or 8 words), one row-kernel launch.  If
 * either problem is large enough for the throughput kernel (large batches), or the two fit neither form, sharing
 * a launch no longer pays and the pair is enqueued as two ordinary launches on `stream`, first then second.
 * abits / wbits / encodings are common to both; everything else is per problem.
 * `first` and `second` are HOST structs, read before the call returns; their pointers are device pointers.
 * The two problems must not write buffers the other reads or writes.
 */
typedef struct dlrt_conv_problem {
    const uint32_t *X;
    const uint32_t *Wp;
    const float *scale; /* may be NULL if only out_acc is given */
    const float *bias;  /* may be NULL */
    int N, H, W, Ci, Co, KH, KW, stride_h, stride_w, pad_h, pad_w;
    int32_t *out_acc;     /* any of the four outputs may be NULL, not all */
    float *out_f32;
    uint8_t *out_q;
    uint32_t *out_packed;
    int qbits;
} dlrt_conv_problem;

dlrt_status dlrt_bitserial_conv2d_fused_pair(const dlrt_conv_problem *first, const dlrt_conv_problem *second,
                                             int abits, int wbits, dlrt_encoding enc_a, dlrt_encoding enc_w,
                                             void *stream);

/*
 * Host-only introspection: which kernel and tile the library would use for a contraction with M outputs
 * rows (conv: N*Ho*Wo), N output columns (conv: Co) and K reduction elements per output, padded per tap as
 * the packed formats are (conv: KH*KW*ceil(Ci/32)*32).  Launches nothing.
 *   *block_kernel = 1: the throughput kernel (one 256-thread block per tile_rows x tile_cols tile, ksplit 1)
 *   *block_kernel = 0: the latency kernel (one wave per tile_rows x 32 tile, ksplit waves split K)
 *   *block_kernel = 2: the row kernel (one output row per lane: a wave covers 64 rows x tile_cols columns);
 *                      taken when the reduction is at most 16 packed words (or 18) and the problem has
 *                      enough 64-row x 32-column waves for that reduction length.  tile_cols is the answer for
 *                      a call that writes only out_packed from unsigned activations (16 columns are possible
 *                      there); any other call gets whole words, at least 32.
 *   *block_kernel = 3: the panel kernel (one output row per lane, 64 rows x tile_cols columns per wave, the
 *                      reduction walked in panels against weights in LDS); taken for long reductions with
 *                      many rows.  The answer assumes 16-byte aligned operands and, for a convolution, a
 *                      channel count that is a multiple of 128; otherwise such a call takes the throughput kernel.
 * Any output pointer may be NULL.
 */
dlrt_status dlrt_query_plan(int64_t M, int64_t N, int64_t K, int abits, int wbits, int *block_kernel,
                            int *tile_rows, int *tile_cols, int *ksplit);

/*
 * Comparison variant, not the bit-serial path: the same integer GEMM as dlrt_bitserial_gemm,
 *   C[m][n] = sum_k A[m][k] * W[n][k]      int32, row-major, leading dimension N,
 * computed on the UNPACKED quantized values (one int8 per element, K-contiguous, any values in
 * [-128, 127]; the 1-4 bit values of Section IV are valid int8) with int8 matrix instructions.  It is
 * the yardstick for the bit-serial kernels of Section V on hardware that can multiply int8 directly.
 * K must be a multiple of 16 (DLRT_ERR_SHAPE otherwise) and A, W 16-byte aligned (DLRT_ERR_ALIGN).
 * Overflow precondition: |sum| < 2^31.
 */
dlrt_status dlrt_unpacked_gemm_i8(const int8_t *A, const int8_t *W, int32_t *C, int64_t M, int64_t N,
                                  int64_t K, void *stream);

/*
 * Second comparison variant, not the bit-serial path: the same integer GEMM on unpacked SIGNED 4-bit values (one
 * per nibble) with the VALU's eight-way dot-product instruction.  Section V's bit-serial sum costs
 * abits * wbits / 16 lane-ops per multiply-add, this instruction 1 / 8 at any width up to 4 bits: the yardstick
 * for where bit-serial arithmetic stops paying on this chip's vector units.
 *   dlrt_pack_nibbles: src int8 [rows][K] with values in [-8, 7] -> dst words [rows][K / 8], element k in bits
 *                      4 (k % 8) .. 4 (k % 8) + 3 of word k / 8 (the low four bits of its two's-complement pattern).
 *   dlrt_unpacked_gemm_i4: C[m][n] = sum_k A[m][k] * W[n][k], int32, row-major, leading dimension N, on such words.
 * K must be a multiple of 32 (DLRT_ERR_SHAPE otherwise) and src, dst, A, W 16-byte aligned (DLRT_ERR_ALIGN).
 */
dlrt_status dlrt_pack_nibbles(const int8_t *src, int64_t rows, int64_t K, uint32_t *dst, void *stream);
dlrt_status dlrt_unpacked_gemm_i4(const uint32_t *A, const uint32_t *W, int32_t *C, int64_t M, int64_t N,
                                  int64_t K, void *stream);

/*
 * Dequantize / requantize epilogue (Section IV: t_hat = t_bar * s, then the quantizer again for
 * the next layer), per output channel:
 *   y = fmaf((float)acc[r][c], scale[c], bias ? bias[c] : 0.0f)          -> out_f32 (may be NULL)
 *   q = (uint8) min(max(rint(y), 0), 2^qbits - 1), ties to even          -> out_q   (may be NULL)
 * acc is rows x C with the channel innermost; out_f32 and out_q must not both be NULL; qbits in
 * 1..8 is read only when out_q is given.
 */
dlrt_status dlrt_epilogue_f32(const int32_t *acc, const float *scale, const float *bias,
                              int64_t rows, int C, float *out_f32, uint8_t *out_q, int qbits,
                              void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DLRT_H */
