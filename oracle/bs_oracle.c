/*
 * CPU oracle for the bit-serial few-bit integer matrix multiply and its feeders.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct C written from the
 * paper's definitions.  It shares no code, header, table or helper with the HIP
 * library and must never be linked or called from the product path; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Everything here is exact integer arithmetic.  Matrices hold *logical values*
 * (bipolar weights are -1/+1, two's-complement w-bit values are
 * -2^(w-1)..2^(w-1)-1, unsigned a-bit values are 0..2^a-1) as int8.
 *
 * Parity pins (tests/test_oracle_*.py): numpy int64 matmul, the bit-plane
 * identity of Sec. 3.1, brute force over every tiny value tuple, closed forms,
 * the K - 2*popcount(XOR) bipolar identity, zero-padding neutrality, the HWGQ
 * worked example of Sec. 2, the ceil-rounding and affine-absorption rules of
 * Sec. 2.1.3, direct convolution against lowering followed by GEMM.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* O1: the product of two few-bit integer matrices by its plain definition    */
/* (Sec. 3.1: "W . A").  W is [M][K], A is [K][N], C is [M][N], all row-major.*/
/* The k loop sits outside the n loop only so that the compiler can vectorise */
/* the innermost statement; every term of the definition is still added once. */
/* ------------------------------------------------------------------------- */
void oracle_gemm_i8(const int8_t *W, const int8_t *A, int32_t *C,
                    int64_t M, int64_t K, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        int32_t *c = C + m * N;
        for (int64_t n = 0; n < N; ++n) c[n] = 0;
        for (int64_t k = 0; k < K; ++k) {
            const int32_t w = W[m * K + k];
            const int8_t *a = A + k * N;
            for (int64_t n = 0; n < N; ++n) c[n] += w * (int32_t)a[n];
        }
    }
}

/* One output element of the same product, in 64-bit, for sampled checks at   */
/* sizes where the full product would take too long on the host.             */
int64_t oracle_dot_i8(const int8_t *W, const int8_t *A,
                      int64_t m, int64_t n, int64_t K, int64_t N)
{
    int64_t s = 0;
    for (int64_t k = 0; k < K; ++k) s += (int64_t)W[m * K + k] * (int64_t)A[k * N + n];
    return s;
}

/* ------------------------------------------------------------------------- */
/* O4: bit-plane packing, one bit at a time (Sec. 3.1: plane i of X is the    */
/* binary matrix of bit i of every element; Alg. 1: depth packed into words). */
/*   X       [rows][depth] logical values                                     */
/*   fmt     0 unsigned: code = v; 1 two's complement: code = v mod 2^bits;   */
/*           2 bipolar (bits == 1): code = (v + 1) / 2                        */
/*   planes  [bits][rows][stride] 64-bit words, bit b of word d <-> k = 64d+b */
/*           (least significant bit first); every bit beyond depth is zero.   */
/* ------------------------------------------------------------------------- */
void oracle_pack(const int32_t *X, int64_t rows, int64_t depth, int bits, int fmt,
                 uint64_t *planes, int64_t stride)
{
    memset(planes, 0, (size_t)bits * (size_t)rows * (size_t)stride * sizeof(uint64_t));
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < depth; ++k) {
            int32_t v = X[r * depth + k];
            uint32_t code;
            if (fmt == 2) code = (uint32_t)((v + 1) / 2);
            else if (fmt == 1) code = (uint32_t)v & ((1u << bits) - 1u);
            else code = (uint32_t)v;
            for (int p = 0; p < bits; ++p)
                if ((code >> p) & 1u)
                    planes[((int64_t)p * rows + r) * stride + k / 64] |= (uint64_t)1 << (k % 64);
        }
}

/* ------------------------------------------------------------------------- */
/* O1b(i): Algorithms 1 and 2 taken step by step on packed planes.            */
/* BinaryGEMM adds alpha * popcount(W(r,d) & A(c,d)) over the depth words;    */
/* BitSerialGEMM calls it once per plane pair with alpha = sgnW*sgnA*2^(i+j), */
/* sgn = -1 only on the most significant plane of an operand declared signed  */
/* (two's complement); an unsigned operand has sgn = +1 on every plane, which */
/* is the unsigned identity of Sec. 3.1.  res is zeroed first (the listing    */
/* shows only the accumulation).                                              */
/* ------------------------------------------------------------------------- */
static void binary_gemm(const uint64_t *W, const uint64_t *A, int64_t *res,
                        int64_t rows, int64_t cols, int64_t depth_words,
                        int64_t wstride, int64_t astride, int64_t alpha)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c)
            for (int64_t d = 0; d < depth_words; ++d)
                res[r * cols + c] += alpha *
                    (int64_t)__builtin_popcountll(W[r * wstride + d] & A[c * astride + d]);
}

/* min_shift > 0 gives the approximate product the paper's conclusion mentions: only the  */
/* plane pairs of weight 2^(i+j) >= 2^min_shift are summed.                                */
void oracle_bitserial_gemm_from(const uint64_t *Wp, int wbits, int wsigned,
                                const uint64_t *Ap, int abits, int asigned,
                                int64_t *res, int64_t rows, int64_t cols,
                                int64_t depth_words, int64_t wstride, int64_t astride, int min_shift);

void oracle_bitserial_gemm(const uint64_t *Wp, int wbits, int wsigned,
                           const uint64_t *Ap, int abits, int asigned,
                           int64_t *res, int64_t rows, int64_t cols,
                           int64_t depth_words, int64_t wstride, int64_t astride)
{
    oracle_bitserial_gemm_from(Wp, wbits, wsigned, Ap, abits, asigned, res, rows, cols, depth_words, wstride, astride, 0);
}

void oracle_bitserial_gemm_from(const uint64_t *Wp, int wbits, int wsigned,
                                const uint64_t *Ap, int abits, int asigned,
                                int64_t *res, int64_t rows, int64_t cols,
                                int64_t depth_words, int64_t wstride, int64_t astride, int min_shift)
{
    for (int64_t i = 0; i < rows * cols; ++i) res[i] = 0;
    for (int i = 0; i < wbits; ++i)
        for (int j = 0; j < abits; ++j) {
            if (i + j < min_shift) continue;
            int64_t sgnW = (wsigned && i == wbits - 1) ? -1 : 1;
            int64_t sgnA = (asigned && j == abits - 1) ? -1 : 1;
            binary_gemm(Wp + (int64_t)i * rows * wstride, Ap + (int64_t)j * cols * astride,
                        res, rows, cols, depth_words, wstride, astride,
                        sgnW * sgnA * ((int64_t)1 << (i + j)));
        }
}

/* ------------------------------------------------------------------------- */
/* O3: convolution by its direct definition (Sec. 3: convolutions between     */
/* feature maps and kernels), never through lowering.                         */
/*   in   [H][W][C]          (HWC, channel fastest)                           */
/*   filt [F][KH][KW][C]                                                      */
/*   out  [OH][OW][F] int32, OH = (H + 2p - KH)/s + 1, same for OW            */
/* Taps that fall outside the image contribute 0.                             */
/* ------------------------------------------------------------------------- */
void oracle_conv_direct(const int8_t *in, const int8_t *filt, int32_t *out,
                        int H, int W, int C, int F, int KH, int KW, int s, int p)
{
    const int OH = (H + 2 * p - KH) / s + 1, OW = (W + 2 * p - KW) / s + 1;
#pragma omp parallel for schedule(static)
    for (int oh = 0; oh < OH; ++oh)
        for (int ow = 0; ow < OW; ++ow)
            for (int f = 0; f < F; ++f) {
                int32_t acc = 0;
                for (int kh = 0; kh < KH; ++kh)
                    for (int kw = 0; kw < KW; ++kw) {
                        const int ih = oh * s + kh - p, iw = ow * s + kw - p;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                        for (int c = 0; c < C; ++c)
                            acc += (int32_t)filt[(((int64_t)f * KH + kh) * KW + kw) * C + c] *
                                   (int32_t)in[((int64_t)ih * W + iw) * C + c];
                    }
                out[((int64_t)oh * OW + ow) * F + f] = acc;
            }
}

/* Plain lowering (im2col, Sec. 3.2) on unpacked values:                      */
/*   L[(kh*KW + kw)*C + c][oh*OW + ow] = in[oh*s+kh-p][ow*s+kw-p][c], else 0. */
void oracle_im2col_plain(const int8_t *in, int8_t *L,
                         int H, int W, int C, int KH, int KW, int s, int p)
{
    const int OH = (H + 2 * p - KH) / s + 1, OW = (W + 2 * p - KW) / s + 1;
    const int64_t ncol = (int64_t)OH * OW;
    for (int kh = 0; kh < KH; ++kh)
        for (int kw = 0; kw < KW; ++kw)
            for (int c = 0; c < C; ++c)
                for (int oh = 0; oh < OH; ++oh)
                    for (int ow = 0; ow < OW; ++ow) {
                        const int ih = oh * s + kh - p, iw = ow * s + kw - p;
                        int8_t v = 0;
                        if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                            v = in[((int64_t)ih * W + iw) * C + c];
                        L[(((int64_t)kh * KW + kw) * C + c) * ncol + (int64_t)oh * OW + ow] = v;
                    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
