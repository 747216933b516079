/*
 * bsgemm -- bit-serial few-bit integer matrix multiply for AMD MI355X (gfx950).
 *
 * C ABI of the library.  The operations are those of "Streamlined Deployment for
 * Quantized Neural Networks" (Umuroglu & Jahre): bit-plane packing (Sec. 3.1),
 * the bit-serial GEMM built from AND-popcount binary GEMMs (Alg. 1 and Alg. 2),
 * successive thresholding as the integer activation (Sec. 2.1.1, 2.1.3) and
 * channel-interleaved lowering of convolutions on packed data (Sec. 3.2).
 *
 * Conventions that hold for every call
 *  - All data pointers are DEVICE pointers.  The caller owns every buffer; the
 *    library never allocates, frees or keeps device memory and has no global
 *    state.
 *  - `stream` is a hipStream_t (NULL = the default stream).  Calls only enqueue
 *    work on that stream and return; results are valid once the stream has
 *    reached that point.
 *  - Every call returns a bs_status and never throws or aborts.  Arguments are
 *    checked on the host before anything is launched; on any error nothing has
 *    been enqueued.
 *  - M = weight rows (output channels), K = depth, N = columns (batch x pixels).
 *
 * Packed format (it crosses this boundary, so it is part of the ABI)
 *  - A matrix X of `rows` x `depth` b-bit values is stored as b bit planes,
 *    uint64_t planes[b][rows][S] with S = bs_words_per_row(depth).
 *  - Bit `t` of word `d` of row `r` of plane `p` is bit p of the code of
 *    X[r][64 d + t] (least significant bit first).  Bits at depth indices >= depth
 *    are ZERO in every plane; consumers rely on it.
 *  - Codes: BS_UNSIGNED v in [0, 2^b): code = v.  BS_TWOS_COMPLEMENT v in
 *    [-2^(b-1), 2^(b-1)): code = v mod 2^b (the top plane carries weight
 *    -2^(b-1), the sign rule of Alg. 2).  BS_BIPOLAR (b must be 1) v in {-1,+1}:
 *    code = (v + 1) / 2.
 *  - Both GEMM operands are depth-contiguous: weights as planes of W [M][K],
 *    activations as planes of A-transposed [N][K] (Alg. 1 indexes A by column).
 *  - S is even, so every packed row starts on a 16-byte boundary; plane buffers
 *    must be 16-byte aligned.
 */
#ifndef BSGEMM_H
#define BSGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BS_OK = 0,
    BS_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, bits out of range, bad enum */
    BS_ERR_UNSUPPORTED = -2,   /* valid but not implemented (e.g. bits > 4) */
    BS_ERR_ALIGNMENT = -3,     /* pointer or leading dimension not aligned as documented */
    BS_ERR_OVERFLOW_RISK = -4, /* an int32 accumulator or a 32-bit index could overflow */
    BS_ERR_LAUNCH = -5         /* the HIP runtime refused the launch */
} bs_status;

typedef enum { BS_UNSIGNED = 0, BS_TWOS_COMPLEMENT = 1, BS_BIPOLAR = 2 } bs_format;
typedef enum { BS_I8 = 0, BS_I32 = 1 } bs_dtype;

/* Row stride S of a packed plane in 64-bit words: ceil(depth/64) rounded up to an
 * even count.  Returns 0 for depth <= 0.  Host-only helper. */
int64_t bs_words_per_row(int64_t depth);

/* Depth of a lowered column (Sec. 3.2): kh * kw * 32 * ceil(C / 32).  Each pixel
 * contributes its channels padded to a 32-bit word.  Host-only helper. */
int64_t bs_lowered_depth(int64_t C, int64_t kh, int64_t kw);

/*
 * Bit-plane packing (Sec. 3.1: plane i holds bit i of every element; Alg. 1:
 * depth packed into machine words).
 *   src     device, `dtype` elements holding logical values.
 *           depth_is_strided == 0: element (r, k) at src[r * ld + k]  (weights, M x K)
 *           depth_is_strided != 0: element (r, k) at src[k * ld + r]  (activations
 *           stored K x N; rows = N; the pack transposes)
 *   ld      leading dimension in elements (>= depth, resp. >= rows)
 *   bits    1..4; fmt as above (BS_BIPOLAR requires bits == 1)
 *   planes  device, uint64_t [bits][rows][bs_words_per_row(depth)], 16-byte
 *           aligned, fully overwritten (padding bits and words written as zero)
 * Values outside the format's range are reduced to their low `bits` bits
 * (bipolar: any v > 0 packs as +1).  Errors: INVALID_ARG, UNSUPPORTED,
 * ALIGNMENT (planes), OVERFLOW_RISK (a plane of more than 2^31 32-bit words), LAUNCH.
 */
bs_status bs_pack_planes(const void *src, bs_dtype dtype, int64_t rows, int64_t depth, int64_t ld,
                         int depth_is_strided, int bits, bs_format fmt, uint64_t *planes, void *stream);

/*
 * Bit-serial GEMM (Alg. 2 over Alg. 1): C = W . A with
 *   C[m][n] = sum_i sum_j sgnW(i) sgnA(j) 2^(i+j) sum_d popcount(Wp[i][m][d] & Ap[j][n][d])
 * sgn = -1 only on the top plane of a BS_TWOS_COMPLEMENT operand; for a
 * BS_BIPOLAR operand (value 2 bit - 1) the algebraically equal popcount form is
 * used, so the result is always the integer product of the logical values.
 *   Wp  device, planes [wbits][M][S], S = bs_words_per_row(K)
 *   Ap  device, planes [abits][N][S]
 *   C   device int32 [M][ldc], ldc >= N, OVERWRITTEN (not accumulated into)
 * Errors: INVALID_ARG; UNSUPPORTED (bits > 4); ALIGNMENT (planes 16 B, C 4 B);
 * OVERFLOW_RISK if K * max|w| * max|a| >= 2^31 - 1 (max|v| of a format: unsigned 2^bits - 1, two's
 * complement 2^(bits-1), bipolar 1: otherwise every result lies inside the int32 range and below INT_MAX, the threshold given to rows past M; partial sums are
 * taken modulo 2^32, which does not change an in-range result) or an operand exceeds 2^31 32-bit
 * words; LAUNCH.
 *
 * Engine (Sec. 4.1.1, 4.2: each layer runs on the faster of a bit-serial and a byte-wise engine).
 * bs_gemm, bs_gemm_threshold and the bs_conv_threshold calls take PACKED PLANES and choose per
 * call, with bs_choose_engine's time model, between the AND-popcount kernels (Alg. 1, 2) and a
 * matrix-core kernel whose loader expands the plane bits to int8 or 4-bit floating-point codes
 * on the way to on-chip memory (nothing unpacked is ever written to device memory, no extra
 * buffer or launch).  All engines return identical results.  bs_gemm_on / bs_gemm_threshold_on
 * take the engine as an argument: BS_ENGINE_BITSERIAL is Alg. 2 as printed, whatever the shape.
 */
bs_status bs_gemm(const uint64_t *Wp, int wbits, bs_format wfmt,
                  const uint64_t *Ap, int abits, bs_format afmt,
                  int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc, void *stream);

typedef enum { BS_ENGINE_BITSERIAL = 0, BS_ENGINE_DENSE_I8 = 1, BS_ENGINE_DENSE_FP4 = 2, BS_ENGINE_AUTO = 3 } bs_engine;

/* bs_gemm on a named engine.  BS_ENGINE_AUTO is bs_gemm.  BS_ENGINE_DENSE_FP4 needs operands whose
 * values are all numbers of the E2M1 format (at most 2 bits, or 3-bit two's complement) and
 * K * max|w| * max|a| < 2^24; a dense engine that cannot take the call returns BS_ERR_UNSUPPORTED
 * (nothing is launched).  Other arguments and errors as bs_gemm. */
bs_status bs_gemm_on(bs_engine engine, const uint64_t *Wp, int wbits, bs_format wfmt,
                     const uint64_t *Ap, int abits, bs_format afmt,
                     int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc, void *stream);

/*
 * Approximate product from the higher-order bits only (the approximate-computing use the
 * paper's conclusion points to): the sum of Alg. 2 restricted to plane pairs with
 * i + j >= min_shift,
 *   C[m][n] = sum_{i+j >= min_shift} sgnW(i) sgnA(j) 2^(i+j) sum_d popcount(Wp[i][m][d] & Ap[j][n][d]).
 * min_shift = 0 is bs_gemm; 0 <= min_shift <= wbits + abits - 2.  With many plane pairs the
 * omitted pairs cost no time.  Operands must be BS_UNSIGNED or BS_TWOS_COMPLEMENT
 * (BS_ERR_UNSUPPORTED otherwise); other arguments and errors as bs_gemm.
 */
bs_status bs_gemm_topbits(const uint64_t *Wp, int wbits, bs_format wfmt,
                          const uint64_t *Ap, int abits, bs_format afmt,
                          int64_t M, int64_t N, int64_t K, int min_shift, int32_t *C, int64_t ldc, void *stream);

/*
 * Successive thresholding (Sec. 2.1.1; integer thresholds per Sec. 2.1.3):
 *   Y[m][n] = number of i < T with C[m][n] >= thr[m][i],  T = 2^obits - 1,
 * written as channel-interleaved bit planes, i.e. packed along m:
 *   Yp  device uint64_t [obits][N][bs_words_per_row(M)], fully overwritten.
 * This is exactly the activation-operand format of bs_gemm (depth = M) and the
 * pixel format of bs_im2col_interleaved.
 *   C   device int32 [M][ldc];  thr  device int32 [M][T] (non-decreasing per row
 *   expected; the count is defined and computed for any order).
 * obits 1..4.  Errors: INVALID_ARG, UNSUPPORTED, ALIGNMENT, LAUNCH.
 */
bs_status bs_threshold_activate(const int32_t *C, int64_t ldc, int64_t M, int64_t N,
                                const int32_t *thr, int obits, uint64_t *Yp, void *stream);

/* bs_gemm followed by bs_threshold_activate in one kernel: the int32 product
 * never leaves the chip.  Arguments as in the two calls above. */
bs_status bs_gemm_threshold(const uint64_t *Wp, int wbits, bs_format wfmt,
                            const uint64_t *Ap, int abits, bs_format afmt,
                            int64_t M, int64_t N, int64_t K,
                            const int32_t *thr, int obits, uint64_t *Yp, void *stream);
/* bs_gemm_threshold on a named engine (see bs_gemm_on). */
bs_status bs_gemm_threshold_on(bs_engine engine, const uint64_t *Wp, int wbits, bs_format wfmt,
                               const uint64_t *Ap, int abits, bs_format afmt,
                               int64_t M, int64_t N, int64_t K,
                               const int32_t *thr, int obits, uint64_t *Yp, void *stream);

/*
 * Channel-interleaved lowering on packed data (Sec. 3.2): one im2col per
 * activation bit, moving whole 32-bit words.
 *   in   device uint64_t [abits][H][W][bs_words_per_row(C)]: per bit position,
 *        per pixel, the channels packed as a depth (what bs_threshold_activate
 *        emits for a layer with C output channels and N = H*W).
 *   out  device uint64_t [abits][OH*OW][bs_words_per_row(Kl)], Kl =
 *        bs_lowered_depth(C, kh, kw), OH = (H + 2 pad - kh)/stride + 1, same for
 *        OW; fully overwritten.  Column (oh, ow) is the concatenation over
 *        (r, s) in kernel-row-major order of the first ceil(C/32) 32-bit words of
 *        pixel (oh*stride + r - pad, ow*stride + s - pad), zero words for taps
 *        outside the image.  Lowered depth index = (r*kw + s) * 32*ceil(C/32) + c.
 * The weight matrix must be packed with the same padded depth order.
 * Errors: INVALID_ARG (sizes, kernel larger than padded image), ALIGNMENT, LAUNCH.
 */
bs_status bs_im2col_interleaved(const uint64_t *in, int abits, int H, int W, int C,
                                int kh, int kw, int stride, int pad, uint64_t *out, void *stream);
/* Batch of B images: in [abits][B][H][W][bs_words_per_row(C)], out [abits][B*OH*OW][bs_words_per_row(Kl)]
 * (column = image * OH*OW + output pixel); everything else as bs_im2col_interleaved (B = 1).
 * The copy moves whole 32-bit words and does not look inside them, so any map whose pixels are runs of 32-bit
 * words can be lowered with it: a feature map already unpacked to E2M1 codes by bs_unpack_planes_fp4 (16 bytes
 * per 32 channels, C a multiple of 32) is a one-plane map of 4 C bit-channels, and its lowering is the
 * [B*OH*OW][Kl / 2 bytes] code matrix that bs_gemm_fp4* takes (call with abits = 1 and 4 C for C). */
bs_status bs_im2col_interleaved_batch(const uint64_t *in, int abits, int B, int H, int W, int C, int kh, int kw,
                                      int stride, int pad, uint64_t *out, void *stream);

/*
 * One quantized convolution layer on packed data, without materialising the lowered
 * matrix: the interleaved lowering of Sec. 3.2 is folded into the operand fetch of the
 * bit-serial GEMM (Alg. 2), and successive thresholding (Sec. 2.1.1) into its epilogue.
 * Equivalent to bs_im2col_interleaved followed by bs_gemm_threshold with M = F,
 * N = OH*OW, K = bs_lowered_depth(C, kh, kw).
 *   in   device uint64_t [abits][H][W][bs_words_per_row(C)], packed HWC planes; afmt must be
 *        BS_UNSIGNED or BS_TWOS_COMPLEMENT (spatial padding is the value 0)
 *   Fp   device, filter planes [wbits][F][bs_words_per_row(Kl)], depth order
 *        (r*kw + s) * 32*ceil(C/32) + c as for bs_im2col_interleaved
 *   thr  device int32 [F][2^obits - 1];  Yp device uint64_t [obits][OH*OW][bs_words_per_row(F)],
 *        i.e. the packed HWC planes of the output feature map, fully overwritten.
 * Errors: INVALID_ARG, UNSUPPORTED (bits > 4, bipolar activations, kh or kw > 127, lowered
 * depth above 65536 bits: use the two-call route), ALIGNMENT, OVERFLOW_RISK, LAUNCH.
 */
bs_status bs_conv_threshold(const uint64_t *in, int abits, bs_format afmt, int H, int W, int C,
                            const uint64_t *Fp, int wbits, bs_format wfmt, int F, int kh, int kw,
                            int stride, int pad, const int32_t *thr, int obits, uint64_t *Yp, void *stream);

/*
 * The same layer for a batch of B images (N = batch x pixels, the columns of Sec. 3.2's lowered
 * matrix for all images side by side): in device uint64_t [abits][B][H][W][bs_words_per_row(C)],
 * Yp device uint64_t [obits][B][OH*OW][bs_words_per_row(F)]; everything else as bs_conv_threshold,
 * which is the case B = 1.
 */
bs_status bs_conv_threshold_batch(const uint64_t *in, int abits, bs_format afmt, int B, int H, int W, int C,
                                  const uint64_t *Fp, int wbits, bs_format wfmt, int F, int kh, int kw,
                                  int stride, int pad, const int32_t *thr, int obits, uint64_t *Yp, void *stream);
/* The same layer on a named engine (see bs_gemm_on; BS_ENGINE_AUTO is bs_conv_threshold_batch): the layer is the product
 * F x Kl x (B OH OW), and the matrix-core kernels gather the lowered columns from the packed map themselves, so no
 * lowered matrix exists on any engine. */
bs_status bs_conv_threshold_batch_on(bs_engine engine, const uint64_t *in, int abits, bs_format afmt, int B, int H, int W,
                                     int C, const uint64_t *Fp, int wbits, bs_format wfmt, int F, int kh, int kw,
                                     int stride, int pad, const int32_t *thr, int obits, uint64_t *Yp, void *stream);

/*
 * Max pooling of a few-bit feature map held as packed HWC planes (unsigned codes).  Not a
 * step of the paper's hot path (pooling is one of its "other layers", Sec. 4.2); provided so
 * that the quantized layers of Table 2 chain without unpacking.  Exact because thresholding
 * is monotone: pooling codes equals thresholding pooled accumulators.
 *   in   device uint64_t [bits][H][W][bs_words_per_row(C)]
 *   out  device uint64_t [bits][OH][OW][bs_words_per_row(C)], OH = (H - k)/stride + 1, no padding
 * Errors: INVALID_ARG (k > H or W), UNSUPPORTED (bits > 4), ALIGNMENT, OVERFLOW_RISK, LAUNCH.
 */
bs_status bs_maxpool_packed(const uint64_t *in, int bits, int H, int W, int C, int k, int stride,
                            uint64_t *out, void *stream);
/* Batch of B maps: in [bits][B][H][W][bs_words_per_row(C)], out [bits][B][OH][OW][bs_words_per_row(C)]. */
bs_status bs_maxpool_packed_batch(const uint64_t *in, int bits, int B, int H, int W, int C, int k, int stride,
                                  uint64_t *out, void *stream);

/*
 * bs_conv_threshold_batch reading its input through a max pooling: the layer sequence pooling -> convolution ->
 * thresholds (AlexNet's pool2 -> conv3 and pool5 -> fc6; Sec. 4.2 runs pooling as a separate layer) in one call.  The
 * pooled map is never written: the kernel that gathers a lowered column (Sec. 3.2) forms every 32-channel word of it as
 * the bit-sliced maximum over its pool_k x pool_k window of the map in memory.  The result equals
 * bs_maxpool_packed_batch followed by bs_conv_threshold_batch bit for bit.
 *   in   device uint64_t [abits][B][H][W][bs_words_per_row(C)], unsigned codes (H x W: the unpooled map)
 *   pool_k, pool_stride  window (1..3) and stride of the pooling; the convolution sees a map of
 *        PH x PW, PH = (H - pool_k) / pool_stride + 1
 *   everything else as bs_conv_threshold_batch with H, W replaced by PH, PW.
 * A kernel that covers the whole pooled map (kh = PH, kw = PW, pad = 0) is a fully connected layer on the flattened
 * pooled map; with at most 4 images it runs on the few-column kernel, which streams the weights once.  All other cases
 * run on the bit-serial kernel with narrow tiles, meant for the small batches where a launch saved matters; for
 * large batches pooling and convolution as two calls are faster (the convolution then goes to the matrix cores).
 * Errors: as bs_conv_threshold_batch; INVALID_ARG also for pool_k < 1 or a window larger than the map;
 * UNSUPPORTED for pool_k > 3.
 */
bs_status bs_pool_conv_threshold_batch(const uint64_t *in, int abits, int B, int H, int W, int C, int pool_k,
                                       int pool_stride, const uint64_t *Fp, int wbits, bs_format wfmt, int F, int kh,
                                       int kw, int stride, int pad, const int32_t *thr, int obits, uint64_t *Yp,
                                       void *stream);

/*
 * Dense engine.  The paper configures each quantized layer to run on either its
 * bit-serial engine or an 8-bit engine (Sec. 4.2) and gives the break-even rule (Sec.
 * 4.1.1).  On this chip the 8-bit matrix cores win the large compute-bound shapes, so the
 * same product C = W . A (Sec. 3.1) is also offered from unpacked int8 operands; the
 * bit-serial calls remain the choice for bandwidth-bound shapes (few columns) and small
 * layers.  bs_choose_engine below makes the choice per layer.
 *
 * bs_unpack_planes: inverse of bs_pack_planes.  planes [bits][rows][bs_words_per_row(depth)]
 *   -> dst int8 [rows][ld], logical values, depth-contiguous; ld a multiple of 16 and
 *   >= depth; bytes from depth up to the next multiple of 16 are written as 0.
 * bs_gemm_i8 / bs_gemm_i8_threshold: W int8 [M][ldw], At int8 [N][lda] (activations
 *   transposed, i.e. depth-contiguous like W), both 16-byte aligned with ldw, lda multiples
 *   of 16 and >= K; bytes between K and the leading dimension are ignored.  Outputs exactly
 *   as bs_gemm (C int32 [M][ldc], overwritten) and bs_gemm_threshold (Yp packed planes).
 * Errors: INVALID_ARG, UNSUPPORTED, ALIGNMENT, OVERFLOW_RISK (K >= 2^17), LAUNCH.
 */
bs_status bs_unpack_planes(const uint64_t *planes, int bits, bs_format fmt, int64_t rows, int64_t depth,
                           int8_t *dst, int64_t ld, void *stream);
bs_status bs_gemm_i8(const int8_t *W, int64_t ldw, const int8_t *At, int64_t lda, int64_t M, int64_t N, int64_t K,
                     int32_t *C, int64_t ldc, void *stream);
bs_status bs_gemm_i8_threshold(const int8_t *W, int64_t ldw, const int8_t *At, int64_t lda, int64_t M, int64_t N,
                               int64_t K, const int32_t *thr, int obits, uint64_t *Yp, void *stream);

/*
 * Dense engine, 4-bit floating-point flavour, for operands of at most 2 bits (any format) and
 * 3-bit two's complement: every such value is a number of the E2M1 format (0, 0.5, 1, 1.5, 2, 3,
 * 4, 6 and their negatives), whose matrix-core instruction runs at twice the int8 rate and half
 * the operand bytes.  Products and partial sums are integers below 2^24, so the fp32 accumulation
 * is exact and the results equal bs_gemm / bs_gemm_threshold bit for bit (the product of Sec. 3.1,
 * the thresholds of Sec. 2.1.1).
 *
 * bs_unpack_planes_fp4: planes [bits][rows][bs_words_per_row(depth)] -> dst uint8 [rows][ld], two
 *   E2M1 codes per byte (sign, two exponent bits, one mantissa bit; low nibble = even depth
 *   index); ld in bytes, a multiple of 16 and >= 16 * ceil(depth / 32); codes from depth up to the
 *   next multiple of 32 are written as +0.  UNSUPPORTED for formats with a value outside E2M1
 *   (3-bit unsigned, every 4-bit format).
 * bs_gemm_fp4 / bs_gemm_fp4_threshold: W [M][ldw], At [N][lda] in that layout (device, 16-byte
 *   aligned, ldw and lda multiples of 16 and >= ceil(K / 2)); bytes beyond ceil(K / 2) are ignored,
 *   and for odd K the high nibble of the last byte must be +0 (bs_unpack_planes_fp4 writes it so).
 *   Outputs exactly as bs_gemm_i8 / bs_gemm_i8_threshold.
 * Errors: INVALID_ARG, UNSUPPORTED, ALIGNMENT, OVERFLOW_RISK (K >= 2^18), LAUNCH.
 */
bs_status bs_unpack_planes_fp4(const uint64_t *planes, int bits, bs_format fmt, int64_t rows, int64_t depth,
                               uint8_t *dst, int64_t ld, void *stream);
bs_status bs_gemm_fp4(const uint8_t *W, int64_t ldw, const uint8_t *At, int64_t lda, int64_t M, int64_t N, int64_t K,
                      int32_t *C, int64_t ldc, void *stream);
bs_status bs_gemm_fp4_threshold(const uint8_t *W, int64_t ldw, const uint8_t *At, int64_t lda, int64_t M, int64_t N,
                                int64_t K, const int32_t *thr, int obits, uint64_t *Yp, void *stream);

/*
 * Streamlining, host side (Sec. 2.1).  HOST pointers, double precision, no GPU work.
 *
 * bs_streamline_collapse (Sec. 2.1.2): collapses, per output channel m, the chain
 *   previous quantizer affine (a_q, b_q) moved past the product, alpha-scaling, batch norm
 *   into y = a[m] x + b[m] of the integer accumulator x = (W x_int)[m]:
 *     a[m] = gamma/sigma * alpha * a_q,  b[m] = gamma/sigma * (alpha * b_q * rowsum_w[m] - mu) + beta.
 *   alpha may be NULL (1); gamma, beta, mu, sigma all NULL (no batch norm) or all given;
 *   rowsum_w[m] = sum_k W[m][k] is needed when b_q != 0.
 * bs_streamline_thresholds (Sec. 2.1.3): thr[m][i] = ceil((t[i] - b[m]) / a[m]) for a[m] > 0, so
 *   that for every integer x  #{i : a x + b >= t[i]} = #{i : x >= thr[m][i]}.  For a[m] < 0 the
 *   channel is marked negate[m] = 1 and the thresholds hold for -x (negate that weight row);
 *   negate == NULL with some a[m] < 0 is BS_ERR_UNSUPPORTED.  a[m] == 0 gives thresholds that
 *   are always / never reached.  Values are clamped to the int32 range.
 *   t [T] is the quantizer's threshold list (Sec. 2.1.1), thr [M][T] row-major.
 */
bs_status bs_streamline_collapse(int64_t M, double a_q, double b_q, const int64_t *rowsum_w, const double *alpha,
                                 const double *gamma, const double *beta, const double *mu, const double *sigma,
                                 double *a, double *b);
bs_status bs_streamline_thresholds(const double *t, int T, const double *a, const double *b, int64_t M,
                                   int32_t *thr, uint8_t *negate);

/*
 * Per-layer engine choice (Sec. 4.1.1 and 4.2 of the paper: bit-serial pays below a break-even
 * precision, and each layer should run on the faster engine).  Host-only, no GPU work.
 * Returns, for a wbits x abits product of shape M x K x N from packed planes, the engine bs_gemm, bs_gemm_threshold
 * take by themselves:
 *   BS_ENGINE_BITSERIAL  the AND-popcount kernels (Alg. 1, 2),
 *   BS_ENGINE_DENSE_FP4  the matrix-core kernel on 4-bit floating-point codes (operands of at most 2 bits and
 *                        K (2^wbits - 1) (2^abits - 1) < 2^24), or
 *   BS_ENGINE_DENSE_I8   the matrix-core kernel on int8 codes (everything else below K = 2^30),
 * whichever is fastest under a time model fitted to measurements on MI355X (microseconds, p = wbits * abits,
 * k = K / 1024, thresholding epilogue included):
 *   bit-serial  N > 16, by the tile the launch takes (t32, t64 = tiles of 32 x 32, 64 x 64 the output needs;
 *               g = 2MNK p / 1e9, e = abits MN / 1e6):
 *                 t32 <= 200   (32 x 8 tiles)             3.03 + 0.206 p + k p (0.155 + 0.113 s) + 1.14 e,
 *                                                         s = ceil(B / 256) - 1 further workgroups per compute unit (B below)
 *                 t32 <= 384   (32 x 16 tiles)            1.98 + 0.492 k p + 5.06 e
 *                 t64 <  512   (32 x 32, depth split)     0.38 + 0.839 g + 3.47 e
 *                 else         (64 x 64)                  1.12 + 0.612 k p + 0.685 g + 0.825 e
 *               5 <= N <= 16: min(3.88 + G (0.69 + 0.2 p + 0.031 p k), 3.64 + R p (0.253 k + 0.21)), with
 *               G = ceil(N / 4) M / 4096 (streaming kernel, groups of four columns), R = 1 + max(0, B - 256) / 900,
 *               B = ceil(M / 32) ceil(N / 8) (tiled kernel, 32 x 8 tiles); bs_gemm itself picks between these two
 *   dense       F + ceil(K / d) r c + E abits MN / 1e6, with d = 256 depth indices per period of the kernel's pipeline
 *               as fp4 codes, 128 as int8 codes; r = rounds of tiles over the chip (bs_planes_tile); and the time of a
 *               period c = c1 + c2 P + f (c3 + c4 P) + c5 max(0, f - h), P = wbits + abits planes to request and merge,
 *               f = the part of the chip's tile slots that is filled (256, 512, 1024 slots for the three tiles), h = 1/2
 *               (1/4 for the 64 x 64 tile): beyond it workgroups share a compute unit; c5 applies to max(0, f - h):
 *                                    F      c1     c2      c3      c4      c5     E
 *                 int8,  64 x 64     4.64   0.613  0.0324       0  0.0248  0.335  0.316
 *                 int8, 128 x 128    5.69   0.753  0.0581  0.0339  0.0303  0.285  0.305
 *                 int8, 256 x 256   11.42   1.054  0.1341       0  0.0738      0  0.191
 *                 fp4,   64 x 64     4.48   0.499  0.0328       0  0.0404  0.320  0.207
 *                 fp4,  128 x 128    5.38   0.602  0.0500  0.0448  0.0321  0.516  0.247
 *                 fp4,  256 x 256    9.29   0.854  0.1456       0  0.0862      0  0.120
 * N <= 4 is always bit-serial (weights are read once, wbits/8 byte per weight, and nothing is expanded).
 * Invalid arguments (bits outside 1..4, bipolar with bits != 1, non-positive sizes) return BS_ENGINE_BITSERIAL.
 */
bs_engine bs_choose_engine(int wbits, bs_format wfmt, int abits, bs_format afmt, int64_t M, int64_t N, int64_t K);

/* Tile edge (256, 128 or 64) the matrix-core kernel on packed planes takes for an M x N output, the rounds of such tiles
 * over the chip (256 slots for the largest tile, 512 and 1024 for the smaller ones) and their number (either pointer may be NULL).
 * Host-only; part of the time model above. */
int bs_planes_tile(int64_t M, int64_t N, long long *rounds, long long *tiles);

/*
 * Diagnostic, not part of the versioned interface (bs_version does not cover it; it may change or go
 * without notice): rate probe for the instruction pair of Alg. 1's inner loop (AND, popcount-accumulate).
 * Launches `workgroups` workgroups of 256 lanes; every lane executes passes * 16 AND and passes * 16
 * popcount-add instructions on registers (no memory traffic, one idle issue slot per pair as in the
 * GEMM's inner loop) and the workgroup stores one word to sink [workgroups] (device memory,
 * caller-owned) so that the work is observable.  passes must be a positive multiple of 4.
 * Lane-operations per launch: workgroups * 256 * passes * 32.  Timed by the caller, it gives the
 * measured ceiling that goes beside the theoretical VALU popcount peak.  Asynchronous on `stream`.
 */
bs_status bs_probe_popcount_rate(uint32_t *sink, int workgroups, int passes, void *stream);

/*
 * Diagnostic, not part of the versioned interface: streaming read of `bytes` bytes (a multiple of 16) from src
 * (device, 16-byte aligned) with 16-byte loads, four in flight per lane, `workgroups` workgroups of 256 lanes each
 * walking 16 KiB slices round-robin; every workgroup XORs what it read into sink [workgroups] (device, caller-owned,
 * not cleared).  non_temporal != 0 reads with the non-temporal hint.  Timed by the caller on a buffer that is not in
 * any cache, it gives the shortest time in which a kernel of this library can bring that many bytes from memory:
 * the measured floor that goes beside the HBM peak for the few-column (batch-1) layers of Table 2.
 */
bs_status bs_probe_stream_read(const void *src, int64_t bytes, uint32_t *sink, int workgroups, int non_temporal,
                               void *stream);

const char *bs_status_string(bs_status s);
int bs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BSGEMM_H */
