/* libdybit: DyBit quantization and DyBit x DyBit matrix products on AMD MI355X (gfx950).
 *
 * C ABI.  Every function returns a dybit_status (or a plain value where said);
 * nothing throws or aborts.  Argument errors are found on the host before any
 * kernel is launched, so they can be exercised on a machine without a GPU.
 *
 * Pointers are tagged [host] or [device].  Device work is asynchronous on the
 * given stream (a raw hipStream_t; NULL is the default stream).  The caller owns
 * every buffer; the library allocates no device memory.
 *
 * Number format (paper Sec. III-A, Eq. 1, Table I).  An N-bit signed code is a
 * sign bit followed by m = N-1 magnitude bits; an N-bit unsigned code is m = N
 * magnitude bits.  Magnitude code c decodes to
 *     0                         c == 0
 *     2^(m-1)                   c all ones (Table I: 1111 -> 8)
 *     c / 2^(m-1)               first bit 0 (fraction only)
 *     2^(i-1) (1 + x / 2^k)     i leading ones, a zero, then k = m-i-1 fraction bits x
 * and a signed code to (-1)^s times that.  The pattern sign=1, magnitude=0 decodes
 * to +0 and is never produced.
 *
 * Packed storage.  Codes form a little-endian bit stream: code j occupies bits
 * [j*bits, (j+1)*bits) of the byte stream, least significant bit first (4-bit:
 * element 2j in the low nibble of byte j; 6-bit: four codes in three bytes).
 * Matrix rows start on a byte boundary, so K*bits must be a multiple of 8.
 */
#ifndef DYBIT_H
#define DYBIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DYBIT_OK = 0,
    DYBIT_ERR_INVALID_ARG = 1,      /* negative or inconsistent size, bad flag value         */
    DYBIT_ERR_UNSUPPORTED_BITS = 2, /* bits not in {2, 4, 6, 8}, or a format with m < 1       */
    DYBIT_ERR_BAD_SCALE = 3,        /* a scale that is not a finite, normal, positive float   */
    DYBIT_ERR_ALIGNMENT = 4,        /* a packed row that does not end on a byte boundary      */
    DYBIT_ERR_NULL = 5,             /* a required pointer is NULL                             */
    DYBIT_ERR_HIP = 6               /* the HIP runtime reported an error at launch            */
} dybit_status;

typedef struct {
    int32_t bits;      /* 2, 4, 6 or 8                                                        */
    int32_t is_signed; /* 1: sign + (bits-1) magnitude bits; 0: bits magnitude bits (Table I) */
} dybit_fmt;

typedef void *dybit_stream; /* a raw hipStream_t */

/* ---- host-only helpers (no GPU needed) ---------------------------------- */

/* Value of every code of a format (Eq. 1, Table I).
 * values_out [host]: 2^bits floats, indexed by the code.  count_out [host, may be NULL]: 2^bits. */
dybit_status dybit_codebook(dybit_fmt f, float *values_out, int32_t *count_out);

/* ceil(n * bits / 8); 0 for an unsupported format. */
size_t dybit_packed_bytes(dybit_fmt f, size_t n);

const char *dybit_status_string(dybit_status s);

/* ---- device entry points -------------------------------------------------- */

/* Per-tensor scale ("precision adjusted at the tensor level", Sec. I):
 * *scale_out = max|x| / 2^(m-1) as a float; NaNs are ignored; 1.0 when the maximum is 0 or n == 0.
 * x [device]: n floats.  scale_out [device]: 1 float, written by the call. */
dybit_status dybit_absmax_scale(const float *x, size_t n, dybit_fmt f, float *scale_out,
                                dybit_stream stream);

/* Encoder (Sec. III-B) with round-to-nearest: codes_out[j] is the code whose value times
 * *scale is nearest to x[j] in exact arithmetic, ties to the even magnitude code.  NaN -> code 0;
 * |x| >= scale * 2^(m-1) (and +-Inf) -> all-ones magnitude; negative x in an unsigned format -> 0;
 * a zero magnitude never carries the sign bit.
 * x [device]: n floats, 16-byte aligned.  scale [device]: 1 float.  codes_out [device]:
 * dybit_packed_bytes(f, n) bytes, 16-byte aligned; unused tail bits of the last byte are zero.
 * If *scale is not a finite normal positive float nothing is written and the asynchronous
 * error flag is set (see dybit_get_last_async_error). */
dybit_status dybit_quantize(const float *x, size_t n, dybit_fmt f, const float *scale,
                            uint8_t *codes_out, dybit_stream stream);

/* dybit_scale_from_absmax and dybit_quantize in one launch, for a tensor whose maximum is already known
 * (a running maximum from the epilogue that produced it): scale = *absmax / 2^(m-1) (1.0 for a maximum of
 * 0), *scale_out = scale for the kernels that follow, codes as dybit_quantize with that scale.
 * absmax [device]: 1 float, >= 0.  scale_out [device]: 1 float, a different word (DYBIT_ERR_INVALID_ARG
 * otherwise).  When n is small enough to leave a remainder kernel, both launches write the same scale. */
dybit_status dybit_quantize_absmax(const float *x, size_t n, dybit_fmt f, const float *absmax, float *scale_out,
                                   uint8_t *codes_out, dybit_stream stream);

/* Decoder (Sec. III-B): y_out[j] = (*scale) * value(code j), one float multiply.
 * codes [device]: packed, 16-byte aligned.  y_out [device]: n floats, 16-byte aligned. */
dybit_status dybit_dequantize(const uint8_t *codes, size_t n, dybit_fmt f, const float *scale,
                              float *y_out, dybit_stream stream);

/* Matrix product with floating-point accumulation (Sec. III-B, systolic-array dataflow):
 *   C[i][j] = (*a_scale)(*w_scale) * sum_k value(A[i][k]) * value(W[j][k])  (+ bias[j])  (ReLU)
 * Products of decoded values are exact; the sum is accumulated in float.
 * A_codes [device]: M rows of K packed codes (row stride K*a_fmt.bits/8 bytes).
 * W_codes [device]: N rows of K packed codes.  Both K-contiguous.
 * a_scale, w_scale [device]: 1 float each.  bias [device]: N floats or NULL.  relu: 0 or 1.
 * C [device]: M rows of ldc floats (ldc >= N), only the first N of each row are written.
 * K*bits must be a multiple of 8 for both operands (DYBIT_ERR_ALIGNMENT otherwise).
 * M, N or K equal to 0 is valid (K == 0 writes bias / zeros). */
dybit_status dybit_gemm(int64_t M, int64_t N, int64_t K,
                        const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                        const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                        const float *bias, int32_t relu,
                        float *C, int64_t ldc, dybit_stream stream);

/* Convolution mapped onto the same matrix product (Sec. IV, "GEMM systolic array"), without
 * materialising the patch matrix: row = (b, ho, wo), column = cout, k = (r, s, cin).
 * X_codes [device]: [B][H][W][Cin] packed along Cin (pixel stride Cin*x_fmt.bits/8 bytes).
 * Wt_codes [device]: [Cout][kh][kw][Cin] packed along (kh, kw, Cin).
 * Y [device]: [B][Ho][Wo][Cout] floats, Ho = (H + 2 pad - kh)/stride + 1 (same for Wo).
 * Taps outside the image contribute exactly 0.  Cin*bits must be a multiple of 8 for both
 * formats (DYBIT_ERR_ALIGNMENT otherwise). */
dybit_status dybit_conv2d(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                          int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                          const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                          const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                          const float *bias, int32_t relu,
                          float *Y, dybit_stream stream);

/* Extended epilogue.  These variants do what dybit_gemm / dybit_conv2d do, with two optional additions:
 *
 *   residual  the identity shortcut of the residual networks the method is evaluated on (Sec. IV,
 *             ResNet-18 / ResNet-50): C = acc * sA sW + bias + residual, then the ReLU.  An fp32
 *             tensor laid out exactly like the output (GEMM: M rows of ldc floats; convolution:
 *             [B][Ho][Wo][Cout]); it must not overlap the output.  NULL: no shortcut.
 *   absmax    write-back support (Sec. III-B: results leave the array as DyBit codes, so with
 *             tensor-level scales the encoder of the next layer needs max|result| first): the maximum
 *             of |value| over the values written (after bias, shortcut and ReLU, NaNs ignored) is
 *             folded into a running maximum, *absmax = max(*absmax, max|C|).  That spares the pass
 *             over C that dybit_absmax_scale would need; finish with dybit_scale_from_absmax.
 *             1 float [device, in/out], non-negative on entry (0 before the first contributing call),
 *             updated with atomic maxima on its bit pattern.  NULL: not tracked.
 *
 * All other arguments: as in dybit_gemm / dybit_conv2d. */
dybit_status dybit_gemm_ex(int64_t M, int64_t N, int64_t K,
                           const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                           const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                           const float *bias, const float *residual, int32_t relu,
                           float *C, int64_t ldc, float *c_absmax, dybit_stream stream);
dybit_status dybit_conv2d_ex(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                             int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                             const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                             const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                             const float *bias, const float *residual, int32_t relu,
                             float *Y, float *y_absmax, dybit_stream stream);

/* Fused write-back (Sec. III-B: the floating-point intermediate results are quantized to DyBit before
 * they are written back).  These variants do what the _ex variants do and, in the same epilogue, encode
 * every result with the format c_fmt and the given scale -- exactly the code dybit_quantize would produce
 * from the fp32 value the call computes -- and store the codes packed like an activation operand of the
 * next layer: M rows of N codes (convolution: [B][Ho][Wo][Cout], packed along Cout).
 *
 *   c_fmt     4-, 6- or 8-bit, signed or unsigned (DYBIT_ERR_UNSUPPORTED_BITS for 2-bit); N * bits must
 *             be a multiple of 32, i.e. rows are whole 32-bit words (DYBIT_ERR_ALIGNMENT otherwise).
 *   c_scale   [device] 1 float, known before the call (a calibrated or previous-iteration scale: the
 *             maximum of this call's results is only known when it ends).  Results beyond
 *             scale * 2^(m-1) saturate to the all-ones magnitude, as in dybit_quantize.  A scale that
 *             is not positive and finite, or lies outside [2^-100, 2^100], writes no codes and sets the
 *             asynchronous error flag (DYBIT_ERR_BAD_SCALE, see dybit_get_last_async_error).
 *   C_codes   [device] M * N * bits / 8 bytes, 4-byte aligned, written by the call; must not overlap
 *             any other argument.  NULL: no codes, the call is the _ex variant.
 *   C / Y     the fp32 output becomes optional: NULL skips it (DYBIT_ERR_NULL when both outputs are
 *             NULL).  ldc still gives the layout of `residual`; ldc and N must be below 2^23.
 *
 * All other arguments: as in dybit_gemm_ex / dybit_conv2d_ex; the running maximum, when asked for, is
 * that of the fp32 values, before encoding. */
dybit_status dybit_gemm_wb(int64_t M, int64_t N, int64_t K,
                           const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                           const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                           const float *bias, const float *residual, int32_t relu,
                           float *C, int64_t ldc, float *c_absmax,
                           dybit_fmt c_fmt, const float *c_scale, uint8_t *C_codes, dybit_stream stream);
dybit_status dybit_conv2d_wb(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                             int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                             const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                             const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                             const float *bias, const float *residual, int32_t relu,
                             float *Y, float *y_absmax,
                             dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream);

/* The write-back variants with the shortcut tensor itself given as DyBit codes (Sec. III-B: between layers
 * the activations exist in memory as codes only; a residual block then adds the codes its input was
 * stored as): C = relu?(A W^T + bias + r_scale * value(R_codes)), encoded as in dybit_gemm_wb.
 *
 *   R_codes   [device] M rows of N codes, packed like C_codes ([B][Ho][Wo][Cout] for the convolution), rows
 *             of N * bits / 8 bytes (N * bits a multiple of 8, DYBIT_ERR_ALIGNMENT otherwise); read only;
 *             must not overlap C_codes.  NULL: DYBIT_ERR_NULL.
 *   r_fmt     4-, 6- or 8-bit, signed or unsigned (DYBIT_ERR_UNSUPPORTED_BITS for 2-bit).
 *   r_scale   [device] 1 float.  The value added is the fp32 number dybit_dequantize would write for the
 *             code, fl(r_scale * value(code)), in the same fp32 addition as the fp32 shortcut of the _wb form.
 *   C_codes   required here (DYBIT_ERR_NULL): the decoder of the shortcut lives in the write-back epilogue.
 *
 * All other arguments and errors: as in dybit_gemm_wb / dybit_conv2d_wb. */
dybit_status dybit_gemm_wb_rc(int64_t M, int64_t N, int64_t K,
                              const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                              const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scale,
                              const float *bias, const uint8_t *R_codes, dybit_fmt r_fmt, const float *r_scale,
                              int32_t relu, float *C, int64_t ldc, float *c_absmax,
                              dybit_fmt c_fmt, const float *c_scale, uint8_t *C_codes, dybit_stream stream);
dybit_status dybit_conv2d_wb_rc(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                                const float *bias, const uint8_t *R_codes, dybit_fmt r_fmt, const float *r_scale,
                                int32_t relu, float *Y, float *y_absmax,
                                dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream);

/* Max pooling on packed DyBit codes (Sec. III-B: between layers the activations exist as codes).  The
 * encoder is monotone, so the maximum by value of a window's codes is the code of the window's maximum: the
 * output equals, bit for bit, dybit_quantize of the pooled fp32 tensor under the scale the input was
 * encoded with (the scale itself is not needed and stays the caller's).
 *
 *   X_codes   [device] [B][H][W][C] codes packed along C, C * bits a multiple of 32 (DYBIT_ERR_ALIGNMENT),
 *             4-byte aligned; read only.
 *   fmt       2-, 4- or 8-bit, signed or unsigned (6-bit: DYBIT_ERR_UNSUPPORTED_BITS).
 *   k, stride, pad   square window; taps outside the image are skipped; 2 * pad <= k and H + 2 pad >= k,
 *             W + 2 pad >= k (DYBIT_ERR_INVALID_ARG otherwise).
 *   Y_codes   [device] [B][Ho][Wo][C] packed the same way, Ho = (H + 2 pad - k) / stride + 1; written by the
 *             call; value zero is always written as the all-zero code.  Must not overlap X_codes. */
dybit_status dybit_maxpool2d_codes(int64_t B, int64_t H, int64_t W, int64_t C,
                                   int32_t k, int32_t stride, int32_t pad,
                                   const uint8_t *X_codes, dybit_fmt fmt, uint8_t *Y_codes, dybit_stream stream);

/* Per-output-channel weight scales (an option on top of the tensor-level scale of Sec. I: one scale per
 * row of W / per filter, the usual remedy for networks whose channels differ widely in range, such as the
 * depthwise-separable ones of Sec. IV).
 *
 * dybit_quantize_rows: max-abs scale and codes of every row of x on its own.
 *   x [device]: rows * cols floats, row-major.  cols * bits must be a multiple of 8 (DYBIT_ERR_ALIGNMENT).
 *   scales_out [device]: rows floats, scales_out[r] = max|x[r][:]| / 2^(m-1) (1.0 for an all-zero row).
 *   codes_out [device]: rows * cols * bits / 8 bytes, rows back to back.  A row whose maximum is infinite
 *   or subnormal gets no codes and sets the asynchronous error flag.
 * dybit_gemm_pc / dybit_conv2d_pc: dybit_gemm_wb / dybit_conv2d_wb with w_scales [device] holding N (Cout)
 *   floats: C[m][n] = sA * w_scales[n] * sum_k a[m][k] w[n][k] (+ bias[n]) (+ residual) (ReLU).  C_codes /
 *   Y_codes may be NULL (then c_fmt and c_scale are ignored and the fp32 output is required). */
dybit_status dybit_quantize_rows(const float *x, int64_t rows, int64_t cols, dybit_fmt f, float *scales_out,
                                 uint8_t *codes_out, dybit_stream stream);
dybit_status dybit_gemm_pc(int64_t M, int64_t N, int64_t K,
                           const uint8_t *A_codes, dybit_fmt a_fmt, const float *a_scale,
                           const uint8_t *W_codes, dybit_fmt w_fmt, const float *w_scales,
                           const float *bias, const float *residual, int32_t relu,
                           float *C, int64_t ldc, float *c_absmax,
                           dybit_fmt c_fmt, const float *c_scale, uint8_t *C_codes, dybit_stream stream);
dybit_status dybit_conv2d_pc(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                             int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                             const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                             const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scales,
                             const float *bias, const float *residual, int32_t relu,
                             float *Y, float *y_absmax,
                             dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream);

/* Depthwise convolution (the layer type of the depthwise-separable network of Sec. IV): every channel is
 * filtered on its own,
 *     Y[b][ho][wo][c] = sX*sW * sum_{r,s} x[b][ho*stride-pad+r][wo*stride-pad+s][c] * w[r][s][c] (+ bias[c]) (ReLU),
 * taps outside the image contributing 0.
 * X_codes [device]: [B][H][W][C] codes;  Wt_codes [device]: [kh][kw][C] codes (channel innermost, like the
 * image); formats of 2, 4 or 8 bits (DYBIT_ERR_UNSUPPORTED_BITS for 6), C * bits a multiple of 32 for both
 * (DYBIT_ERR_ALIGNMENT), buffers 16-byte aligned.  x_scale, w_scale [device]: 1 float each.
 * bias [device, may be NULL]: C floats.  Y [device]: [B][Ho][Wo][C] floats.  y_absmax [device, may be NULL]:
 * running maximum as in dybit_gemm_ex.  Filters and strides whose input patch for 8 x 8 outputs exceeds
 * 64 KiB of floats for 32 channels (e.g. 9 x 9 at stride 4) are refused with DYBIT_ERR_INVALID_ARG. */
dybit_status dybit_dwconv2d(int64_t B, int64_t H, int64_t W, int64_t C,
                            int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                            const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                            const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale,
                            const float *bias, int32_t relu, float *Y, float *y_absmax, dybit_stream stream);

/* dybit_dwconv2d with the options of the matrix-product calls (Sec. IV's depthwise-separable network inside
 * the write-back dataflow of Sec. III-B):
 *   w_per_channel  1: w_scale [device] holds C floats, one per channel (the scales dybit_quantize_cols
 *                  returns for a [kh*kw][C] filter); 0: one float for the whole filter.
 *   Y              [device, may be NULL when Y_codes is given]: the fp32 output.
 *   y_fmt, y_scale, Y_codes  [may be NULL: no codes]: every result is also encoded with format y_fmt (4 or
 *                  8 bits; DYBIT_ERR_UNSUPPORTED_BITS otherwise) under the known scale *y_scale [device], exactly
 *                  as dybit_quantize would encode the fp32 value, and stored packed along C as [B][Ho][Wo][C]
 *                  codes (C * bits a multiple of 32).  An unusable scale (see dybit_gemm_wb) writes no codes
 *                  and sets the asynchronous error flag.
 * Everything else as in dybit_dwconv2d. */
dybit_status dybit_dwconv2d_wb(int64_t B, int64_t H, int64_t W, int64_t C,
                               int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                               const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                               const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale, int32_t w_per_channel,
                               const float *bias, int32_t relu, float *Y, float *y_absmax,
                               dybit_fmt y_fmt, const float *y_scale, uint8_t *Y_codes, dybit_stream stream);

/* Grouped convolution (the layer type between the dense and the depthwise convolution in the networks of
 * Sec. IV): input and output channels are split into `groups` equal parts and part g of the output sees
 * part g of the input only; output channel n belongs to group n / (Cout / groups).
 * X_codes [device]: [B][H][W][Cin] codes.  Wt_codes [device]: [Cout][kh][kw][Cin / groups] codes.
 * groups must divide Cin and Cout (DYBIT_ERR_INVALID_ARG); a group's channels must start on a byte of every
 * pixel and filter, i.e. (Cin / groups) * bits a multiple of 8 for both formats (DYBIT_ERR_ALIGNMENT).
 * w_scale [device]: 1 float, or Cout floats when w_per_channel is 1.  bias [device, may be NULL]: Cout floats.
 * residual [device, may be NULL]: like Y.  Y [device]: [B][Ho][Wo][Cout] floats.  y_absmax: as in dybit_conv2d_ex.
 * One launch per group on the group's channel slices (groups = Cin = Cout is a depthwise convolution with the
 * filters laid out [C][kh][kw][1]; dybit_dwconv2d, with channel-innermost filters, is the fast form of that). */
dybit_status dybit_group_conv2d(int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                int32_t kh, int32_t kw, int32_t stride, int32_t pad, int32_t groups,
                                const uint8_t *X_codes, dybit_fmt x_fmt, const float *x_scale,
                                const uint8_t *Wt_codes, dybit_fmt w_fmt, const float *w_scale, int32_t w_per_channel,
                                const float *bias, const float *residual, int32_t relu,
                                float *Y, float *y_absmax, dybit_stream stream);

/* Max-abs scale and codes of every column of x on its own: the per-channel scales of a depthwise filter,
 * whose layout [kh*kw][C] has the channel innermost.
 *   x [device]: rows * cols floats, row-major.  cols * bits must be a multiple of 8 (DYBIT_ERR_ALIGNMENT).
 *   scales_out [device]: cols floats, scales_out[c] = max|x[:][c]| / 2^(m-1) (1.0 for an all-zero column).
 *   codes_out [device]: rows * cols * bits / 8 bytes, laid out like x.  A column whose maximum is infinite
 *   or subnormal gets code 0 throughout and sets the asynchronous error flag. */
dybit_status dybit_quantize_cols(const float *x, int64_t rows, int64_t cols, dybit_fmt f, float *scales_out,
                                 uint8_t *codes_out, dybit_stream stream);

/* dybit_quantize of a row-major matrix with every row padded with zero codes: row r of x holds `cols` floats,
 * row r of codes_out `cols_padded` codes, of which the last cols_padded - cols are code 0 (value 0).  For a
 * few-channel image whose pixels must end on a byte or word boundary for the convolution (3 -> 4 channels): the
 * codes equal those of dybit_quantize on the zero-padded fp32 tensor, which then need not exist.
 *   x [device]: rows * cols floats.  scale [device]: 1 float, as for dybit_quantize (an unusable scale writes
 *   nothing and sets the asynchronous error flag); padding changes no maximum, so dybit_absmax_scale of x serves.
 *   cols_padded: >= cols, a multiple of 4 (DYBIT_ERR_ALIGNMENT).  codes_out [device]: rows * cols_padded * bits / 8
 *   bytes, written by the call. */
dybit_status dybit_quantize_pad(const float *x, int64_t rows, int64_t cols, int64_t cols_padded, dybit_fmt f,
                                const float *scale, uint8_t *codes_out, dybit_stream stream);

/* *scale_out = *absmax / 2^(m-1), or 1.0 when *absmax == 0: the last step of dybit_absmax_scale,
 * for a maximum obtained otherwise.  absmax, scale_out [device]: 1 float each (may be the same word). */
dybit_status dybit_scale_from_absmax(const float *absmax, dybit_fmt f, float *scale_out, dybit_stream stream);

/* Quantize and decode again in one pass, y = s * value(code nearest to x / s): the forward of the
 * quantization-aware training step that follows the search (Sec. III-C); bit for bit the result of
 * dybit_dequantize on dybit_quantize's codes, without the codes reaching memory (its gradient:
 * dybit_fake_quant_bwd).
 * x, y_out [device]: n floats each, 16-byte aligned (may be the same buffer).  scale [device]: as for
 * dybit_quantize; an unusable scale writes nothing and sets the asynchronous error flag. */
dybit_status dybit_fake_quant(const float *x, size_t n, dybit_fmt f, const float *scale, float *y_out,
                              dybit_stream stream);

/* Backward of dybit_fake_quant under the straight-through estimator (the fine-tuning step of Sec. III-C
 * treats the rounding as the identity and the saturation as the clamp it is):
 *     grad_in[j] = grad_out[j]  if x[j] lies in [-s vmax, s vmax] (unsigned formats: [0, s vmax]), bounds included,
 *                = 0            otherwise, and for a NaN x[j].
 * x, grad_out, grad_in [device]: n floats each, 16-byte aligned (grad_in may be grad_out).  scale [device]:
 * the scale of the forward; not positive or not finite: nothing is written and the asynchronous error flag is set. */
dybit_status dybit_fake_quant_bwd(const float *x, const float *grad_out, size_t n, dybit_fmt f, const float *scale,
                                  float *grad_in, dybit_stream stream);

/* Quantization error of one tensor in one format (Sec. III-C, Eq. 2):
 *     RMSE = sqrt( mean( ((x - x_hat) / sigma)^2 ) ),   x_hat = s * value(code nearest to x / s),
 * sigma the standard deviation of x (population form, one value for the tensor).  One pass over x.
 * x [device]: n floats, 16-byte aligned, n >= 1 (DYBIT_ERR_INVALID_ARG for 0).  scale [device]: 1 float;
 * a scale that is not positive and finite, or outside [2^-100, 2^100], gives NaN results and sets the
 * asynchronous error flag (DYBIT_ERR_BAD_SCALE).  out [device]: 4 doubles, 8-byte aligned:
 *     out[0] = RMSE, out[1] = sum (x - x_hat)^2, out[2] = sum x, out[3] = sum x^2
 * (the three sums are what devices holding parts of one tensor would add up before the last step).
 * The differences are formed in float (one rounding each), the sums in double; the order of the
 * additions across workgroups is not fixed, so the last bits can differ from call to call.  A NaN
 * or infinity in x gives non-finite results; a constant tensor (sigma = 0) gives inf or NaN. */
dybit_status dybit_rmse(const float *x, size_t n, dybit_fmt f, const float *scale, double *out, dybit_stream stream);

/* Layer-wise bitwidth search (Sec. III-C, Eq. 3, Eq. 4, Alg. 1).  Host only; all pointers [host].
 * Widths are chosen from {8, 4, 2} ("levels" 0, 1, 2).
 *   lat      n_layers * 3 * 3 doubles, lat[(l*3 + w_level)*3 + a_level] > 0: latency of layer l in that mode
 *            (measured on the device, where the paper asks a simulator of its accelerator).
 *   rmse_w   n_layers * 3 doubles >= 0: error (Eq. 2) of layer l's weight tensor at each level.
 *   rmse_a   the same for the layer's input activation tensor.  A layer's error is the sum of the two.
 *   strategy DYBIT_SEARCH_SPEEDUP: least error subject to  total latency at (8,8) / total latency >= constraint
 *            (Eq. 3); DYBIT_SEARCH_RMSE: least latency subject to  total error / total error at (8,8) <=
 *            constraint (Eq. 4).
 *   k        how many layers one round considers (>= 1).
 * Each round takes the layers that can still be lowered, ranks them by the constrained quantity under the
 * current assignment (speedup: slowest first; error: least error first), keeps the first k, re-ranks
 * those by the other quantity (least error first / slowest first; ties to the lower index throughout),
 * and lowers first the weights, then the activations of the listed layers by one level each, checking
 * the ratio after every single step.  Speedup strategy: stops as soon as the ratio reaches the
 * constraint, or when every layer is at 2/2 bits (*met_out = 0).  Error strategy: the constraint is a
 * budget; the first step that exceeds it is taken back and ends the search.
 *   w_bits_out, a_bits_out   n_layers ints each: 8, 4 or 2.  ratio_out, met_out [may be NULL]: the final
 *            ratio and whether it satisfies the constraint.
 * DYBIT_ERR_INVALID_ARG: n_layers < 1, k < 1, unknown strategy, NaN constraint, a latency that is not
 * positive and finite, an error that is negative or not finite, or a zero (8,8) total. */
#define DYBIT_SEARCH_SPEEDUP 0
#define DYBIT_SEARCH_RMSE 1
dybit_status dybit_search(int32_t n_layers, const double *lat, const double *rmse_w, const double *rmse_a,
                          int32_t strategy, double constraint, int32_t k,
                          int32_t *w_bits_out, int32_t *a_bits_out, double *ratio_out, int32_t *met_out);

/* Waits for `stream`, then reports and clears the asynchronous error flag of the current
 * device: *flag_out [host] is DYBIT_OK or DYBIT_ERR_BAD_SCALE (a dybit_quantize kernel since the
 * last call, or a write-back epilogue, found an unusable scale and wrote no codes). */
dybit_status dybit_get_last_async_error(int32_t *flag_out, dybit_stream stream);

/* A caller-owned error word for the calling host thread (for callers that run several streams at once and
 * want to know which one met the error; the library's own flag is one word per device).
 *   device_word [device]: one int32, 4-byte aligned (DYBIT_ERR_ALIGNMENT), zeroed by the caller.  From this
 *   call on, kernels launched by this host thread's calls store DYBIT_ERR_BAD_SCALE there instead of into
 *   the library's flag; the caller reads and clears it (after synchronising with the stream it used) and keeps
 *   it alive until those kernels have finished.  NULL: back to the library's flag.
 * dybit_get_last_async_error keeps reporting the library's flag only.  Host only, no device work. */
dybit_status dybit_set_async_error_word(int32_t *device_word);

/* Which kernel a matrix-product call ran on (Sec. III-B's array has one datapath; this library picks
 * among several kernels by shape and formats).  Host only, no device work.
 *
 * dybit_last_gemm_kernel: the kernel that the calling host thread's most recent dybit_gemm* /
 * dybit_conv2d* call launched (DYBIT_KERNEL_NONE before the first, or when the call returned early:
 * an error, M == 0 or N == 0).
 *
 * dybit_set_option: overrides the automatic choice for the whole process, for tests and A/B
 * measurements.  name / value [host, NUL-terminated]:
 *   "gemm_kernel"  "auto" | "general" | "mid" | "large" | "ws"  -- takes the named kernel family whenever
 *                  the problem meets its preconditions (otherwise the automatic choice continues, which
 *                  dybit_last_gemm_kernel shows)
 *   "gemm_mfma"    "auto" | "f16"   -- "f16" keeps pairs of 4- and 2-bit operands off the e4m3 kernels
 *   "mid_tile"     "auto" | "64" | "128"   -- tile of the e4m3 kernel when it is not the 256 x 256 one
 *   "mid_kgroups"  "auto" | "1" | "2"      -- k-groups per workgroup of the 128 x 128 kernels
 *   "gemm_ws"      "auto" | "off"   -- "off" leaves the weight-stationary kernel out of the automatic choice
 * Initial values come from the environment, read once when the library is first used (DYBIT_GEMM_KERNEL,
 * DYBIT_GEMM_MFMA, DYBIT_MID_TILE, DYBIT_MID_KGROUPS, DYBIT_GEMM_WS=0).  DYBIT_ERR_NULL for a NULL
 * argument, DYBIT_ERR_INVALID_ARG for an unknown name or value.  Not synchronised with calls running on
 * other host threads: set options before starting them. */
typedef enum {
    DYBIT_KERNEL_NONE = 0,
    DYBIT_KERNEL_GENERAL = 1,        /* any formats and shapes, LDS look-up tables, 128 x 128 tile      */
    DYBIT_KERNEL_F16_256 = 2,        /* fp16 MFMA, 256 x 256 tile                                       */
    DYBIT_KERNEL_F16_128_KG1 = 3,    /* fp16 MFMA, 128 x 128 tile, one k-group                          */
    DYBIT_KERNEL_F16_128_KG2 = 4,    /* fp16 MFMA, 128 x 128 tile, two k-groups                         */
    DYBIT_KERNEL_F16_128_ROWS = 5,   /* fp16 MFMA, 128 x 128 tile, few-channel convolution by filter rows */
    DYBIT_KERNEL_F16_WS = 6,         /* fp16 MFMA, weight-stationary                                    */
    DYBIT_KERNEL_F8_256 = 7,         /* e4m3 MFMA, 256 x 256 tile                                       */
    DYBIT_KERNEL_F8_128_KG1 = 8,     /* e4m3 MFMA, 128 x 128 tile, one k-group                          */
    DYBIT_KERNEL_F8_128_KG2 = 9,     /* e4m3 MFMA, 128 x 128 tile, two k-groups                         */
    DYBIT_KERNEL_F8_64 = 10,         /* e4m3 MFMA, 64 x 64 tile, two k-groups                           */
    DYBIT_KERNEL_F8_WS = 11          /* e4m3 MFMA, weight-stationary                                    */
} dybit_kernel_id;
int32_t dybit_last_gemm_kernel(void);
dybit_status dybit_set_option(const char *name, const char *value);

/* Measurement aid, not part of the method: runs only fp16 MFMA instructions (the instruction
 * dybit_gemm uses) on operand values taken from `operands` and reports how many flops the launch
 * performs, so that a caller can time it and obtain the matrix-core rate this device sustains.
 * operands [device]: 9 * 512 * 8 halves (73,728 bytes), 16-byte aligned.  workgroups: grid size
 * (512 threads each).  iters: loop count per wave.  sink [device]: 1 float.  flops_out [host, may
 * be NULL]. */
dybit_status dybit_diag_mfma_f16(const void *operands, int32_t workgroups, int32_t iters,
                                 float *sink, double *flops_out, dybit_stream stream);

/* The same for the fp8 (e4m3) MFMA instruction that pairs of 4-bit formats run on.
 * operands [device]: 9 * 512 * 32 bytes (147,456 bytes) of e4m3 values, 16-byte aligned. */
dybit_status dybit_diag_mfma_f8(const void *operands, int32_t workgroups, int32_t iters,
                                float *sink, double *flops_out, dybit_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* DYBIT_H */
