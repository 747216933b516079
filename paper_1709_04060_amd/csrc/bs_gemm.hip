// Host side of the bit-serial GEMM entry points: argument checks, the per-plane
// coefficients of Alg. 2 (and of the bipolar popcount form), and dispatch on the number
// of weight planes.  The kernel itself lives in bs_gemm_kernel.h.
#include "bs_gemm_kernel.h"

namespace bs {
extern template bs_status launch_wb<1>(const GemmParams &, int, bool, bool, bool, bool, hipStream_t);
extern template bs_status launch_wb<2>(const GemmParams &, int, bool, bool, bool, bool, hipStream_t);
extern template bs_status launch_wb<3>(const GemmParams &, int, bool, bool, bool, bool, hipStream_t);
extern template bs_status launch_wb<4>(const GemmParams &, int, bool, bool, bool, bool, hipStream_t);
}

namespace {
using namespace bs;

void set_coefficients(GemmParams &g, int wbits, bs_format wfmt, int abits, bs_format afmt, int64_t K)
{
    int cw[4] = {0, 0, 0, 0}, ca[4] = {0, 0, 0, 0};
    int ow = 0, oa = 0;
    for (int i = 0; i < wbits; ++i) cw[i] = (wfmt == BS_TWOS_COMPLEMENT && i == wbits - 1) ? -(1 << i) : (1 << i);
    for (int j = 0; j < abits; ++j) ca[j] = (afmt == BS_TWOS_COMPLEMENT && j == abits - 1) ? -(1 << j) : (1 << j);
    if (wfmt == BS_BIPOLAR) { cw[0] = 2; ow = -1; }
    if (afmt == BS_BIPOLAR) { ca[0] = 2; oa = -1; }
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) g.coef[i * 4 + j] = cw[i] * ca[j];
    for (int i = 0; i < 4; ++i) { g.crow[i] = oa * cw[i]; g.ccol[i] = ow * ca[i]; }
    g.c0 = ow * oa * (int)K;
}

bs_status dispatch_wb(const GemmParams &g, int wbits, int abits, bool fuse, bool corr, bool conv, bool xr, hipStream_t st)
{
    switch (wbits) {
    case 1: return launch_wb<1>(g, abits, fuse, corr, conv, xr, st);
    case 2: return launch_wb<2>(g, abits, fuse, corr, conv, xr, st);
    case 3: return launch_wb<3>(g, abits, fuse, corr, conv, xr, st);
    default: return launch_wb<4>(g, abits, fuse, corr, conv, xr, st);
    }
}

// |result| <= K * max|w| * max|a| must fit int32 (sums inside the kernels are taken modulo 2^32, which leaves an
// in-range result unchanged).  The approximate mode sums a subset of the plane pairs, bounded by the unsigned ranges.
bool result_may_overflow(int64_t K, int wbits, bs_format wfmt, int abits, bs_format afmt, bool subset_of_pairs)
{
    const int64_t mw = subset_of_pairs ? (int64_t(1) << wbits) - 1 : bs::max_abs(wbits, wfmt);
    const int64_t ma = subset_of_pairs ? (int64_t(1) << abits) - 1 : bs::max_abs(abits, afmt);
    const int64_t lim = int64_t(1) << 31;
    // (lim - 1: no result reaches INT_MAX, the threshold that rows past M are given)
    return K >= lim || K * mw * ma >= lim - 1;
}

bs_status gemm_common(bs_engine engine, const uint64_t *Wp, int wbits, bs_format wfmt, const uint64_t *Ap, int abits,
                      bs_format afmt, int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc,
                      const int32_t *thr, int obits, uint64_t *Yp, bool fuse, void *stream, int min_shift = 0)
{
    if (engine != BS_ENGINE_BITSERIAL && engine != BS_ENGINE_DENSE_I8 && engine != BS_ENGINE_DENSE_FP4 &&
        engine != BS_ENGINE_AUTO)
        return BS_ERR_INVALID_ARG;
    if (!Wp || !Ap || M <= 0 || N <= 0 || K <= 0) return BS_ERR_INVALID_ARG;
    if (bs_status s = bs::check_bits_fmt(wbits, wfmt)) return s;
    if (bs_status s = bs::check_bits_fmt(abits, afmt)) return s;
    if (!bs::aligned(Wp, 16) || !bs::aligned(Ap, 16)) return BS_ERR_ALIGNMENT;
    if (fuse) {
        if (!thr || !Yp) return BS_ERR_INVALID_ARG;
        if (obits < 1) return BS_ERR_INVALID_ARG;
        if (obits > bs::kMaxBits) return BS_ERR_UNSUPPORTED;
        if (!bs::aligned(thr, 4) || !bs::aligned(Yp, 16)) return BS_ERR_ALIGNMENT;
    } else {
        if (!C || ldc < N) return BS_ERR_INVALID_ARG;
        if (!bs::aligned(C, 4)) return BS_ERR_ALIGNMENT;
    }
    if (result_may_overflow(K, wbits, wfmt, abits, afmt, min_shift > 0)) return BS_ERR_OVERFLOW_RISK;
    const int64_t S = bs_words_per_row(K);
    const int64_t lim = int64_t(1) << 31;
    if (wbits * M * S * 2 >= lim || abits * N * S * 2 >= lim || M >= lim || N >= lim) return BS_ERR_OVERFLOW_RISK;

    GemmParams g{};
    g.W = reinterpret_cast<const uint32_t *>(Wp);
    g.A = reinterpret_cast<const uint32_t *>(Ap);
    g.M = (int)M; g.N = (int)N; g.Kd = (int)(2 * S);
    set_coefficients(g, wbits, wfmt, abits, afmt, K);
    if (min_shift > 0) {  // approximate mode: only plane pairs of weight 2^(i+j) >= 2^min_shift contribute
        if (wfmt == BS_BIPOLAR || afmt == BS_BIPOLAR) return BS_ERR_UNSUPPORTED;
        for (int i = 0; i < 4; ++i)
            for (int j = 0; j < 4; ++j)
                if (i + j < min_shift) g.coef[i * 4 + j] = 0;
    }
    g.C = C; g.ldc = ldc;
    g.thr = thr; g.obits = obits; g.T = fuse ? (1 << obits) - 1 : 0;
    g.Y = reinterpret_cast<uint32_t *>(Yp);
    g.Yd = (int)(2 * bs_words_per_row(M));
    // Both operands bipolar (the W1A1 case of Sec. 3.1): XOR-popcount, dot = K - 2 popcount(XOR)
    const bool xr = (wfmt == BS_BIPOLAR) && (afmt == BS_BIPOLAR);
    if (xr) {
        for (int i = 0; i < 16; ++i) g.coef[i] = 0;
        g.coef[0] = -2;
        g.c0 = (int)K;
        for (int i = 0; i < 4; ++i) g.crow[i] = g.ccol[i] = 0;
    }
    const bool corr = !xr && ((wfmt == BS_BIPOLAR) || (afmt == BS_BIPOLAR));
    g.stream_weights = (long long)wbits * M * S * 8 >= kStreamWeightBytes;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Engine (Sec. 4.1.1, 4.2): the approximate mode exists bit-serially only; otherwise the caller's engine, or the
    // one the time model expects to be fastest for this shape.
    if (min_shift == 0 && engine != BS_ENGINE_BITSERIAL) {
        const bs_engine e = engine == BS_ENGINE_AUTO ? bs_choose_engine(wbits, wfmt, abits, afmt, M, N, K) : engine;
        if (e != BS_ENGINE_BITSERIAL) {
            PlanesGemm q{};
            q.W = g.W; q.A = g.A; q.wbits = wbits; q.abits = abits; q.wfmt = wfmt; q.afmt = afmt;
            q.M = g.M; q.N = g.N; q.K = K; q.Kd = g.Kd;
            q.C = C; q.ldc = ldc; q.thr = thr; q.obits = obits; q.Y = g.Y; q.Yd = g.Yd;
            return launch_planes_mfma(q, e == BS_ENGINE_DENSE_FP4, fuse, st);
        }
    }
    if (gemv_applicable(g, wbits, abits, afmt == BS_BIPOLAR, wfmt == BS_BIPOLAR)) return launch_gemv(g, wbits, abits, fuse, xr, st);
    return dispatch_wb(g, wbits, abits, fuse, corr, false, xr, st);
}

}  // namespace

extern "C" bs_status bs_gemm(const uint64_t *Wp, int wbits, bs_format wfmt, const uint64_t *Ap, int abits,
                             bs_format afmt, int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc, void *stream)
{
    return gemm_common(BS_ENGINE_AUTO, Wp, wbits, wfmt, Ap, abits, afmt, M, N, K, C, ldc, nullptr, 0, nullptr, false, stream);
}

extern "C" bs_status bs_gemm_on(bs_engine engine, const uint64_t *Wp, int wbits, bs_format wfmt, const uint64_t *Ap,
                                int abits, bs_format afmt, int64_t M, int64_t N, int64_t K, int32_t *C, int64_t ldc,
                                void *stream)
{
    return gemm_common(engine, Wp, wbits, wfmt, Ap, abits, afmt, M, N, K, C, ldc, nullptr, 0, nullptr, false, stream);
}

extern "C" bs_status bs_gemm_threshold_on(bs_engine engine, const uint64_t *Wp, int wbits, bs_format wfmt,
                                          const uint64_t *Ap, int abits, bs_format afmt, int64_t M, int64_t N, int64_t K,
                                          const int32_t *thr, int obits, uint64_t *Yp, void *stream)
{
    return gemm_common(engine, Wp, wbits, wfmt, Ap, abits, afmt, M, N, K, nullptr, 0, thr, obits, Yp, true, stream);
}

extern "C" bs_status bs_gemm_threshold(const uint64_t *Wp, int wbits, bs_format wfmt, const uint64_t *Ap, int abits,
                                       bs_format afmt, int64_t M, int64_t N, int64_t K, const int32_t *thr,
                                       int obits, uint64_t *Yp, void *stream)
{
    return gemm_common(BS_ENGINE_AUTO, Wp, wbits, wfmt, Ap, abits, afmt, M, N, K, nullptr, 0, thr, obits, Yp, true, stream);
}

namespace {

// Convolution by implicit lowering, optionally reading its input through a max pooling of pool_k x pool_k windows
// (pool_k = 0: none): H x W is the map in memory, PH x PW the map the convolution sees.
bs_status conv_common(bs_engine engine, const uint64_t *in, int abits, bs_format afmt, int B, int H, int W, int C, int pool_k,
                      int pool_stride, const uint64_t *Fp, int wbits, bs_format wfmt, int F, int kh, int kw, int stride,
                      int pad, const int32_t *thr, int obits, uint64_t *Yp, void *stream)
{
    if (engine != BS_ENGINE_BITSERIAL && engine != BS_ENGINE_DENSE_I8 && engine != BS_ENGINE_DENSE_FP4 &&
        engine != BS_ENGINE_AUTO)
        return BS_ERR_INVALID_ARG;
    if (!in || !Fp || !thr || !Yp || B <= 0 || H <= 0 || W <= 0 || C <= 0 || F <= 0 || kh <= 0 || kw <= 0 ||
        stride <= 0 || pad < 0 || obits < 1)
        return BS_ERR_INVALID_ARG;
    if (bs_status s = bs::check_bits_fmt(wbits, wfmt)) return s;
    if (bs_status s = bs::check_bits_fmt(abits, afmt)) return s;
    // spatial padding is written as zero words, which is the value 0 only for these formats
    if (afmt == BS_BIPOLAR) return BS_ERR_UNSUPPORTED;
    if (obits > bs::kMaxBits) return BS_ERR_UNSUPPORTED;
    int PH = H, PW = W;
    if (pool_k > 0) {
        if (pool_stride <= 0 || pool_k > H || pool_k > W) return BS_ERR_INVALID_ARG;
        // the maximum is taken on the codes, which is the maximum of the values for unsigned codes only; the kernels
        // hold the taps of one window in registers, up to 3 x 3
        if (afmt != BS_UNSIGNED || pool_k > 3) return BS_ERR_UNSUPPORTED;
        PH = (H - pool_k) / pool_stride + 1;
        PW = (W - pool_k) / pool_stride + 1;
    }
    if (PH + 2 * pad < kh || PW + 2 * pad < kw) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(in, 16) || !bs::aligned(Fp, 16) || !bs::aligned(Yp, 16) || !bs::aligned(thr, 4))
        return BS_ERR_ALIGNMENT;
    const int64_t Kl = bs_lowered_depth(C, kh, kw);
    const int64_t S = bs_words_per_row(Kl);
    const int OH = (PH + 2 * pad - kh) / stride + 1, OW = (PW + 2 * pad - kw) / stride + 1;
    const int64_t N = (int64_t)B * OH * OW;
    if (2 * S > kConvMaxLut || kh > 127 || kw > 127) return BS_ERR_UNSUPPORTED;
    if (result_may_overflow(Kl, wbits, wfmt, abits, afmt, false)) return BS_ERR_OVERFLOW_RISK;
    const int64_t lim = int64_t(1) << 31;
    const int64_t pix = 2 * bs_words_per_row(C);
    if (wbits * (int64_t)F * S * 2 >= lim || abits * (int64_t)B * H * W * pix >= lim || N >= lim)
        return BS_ERR_OVERFLOW_RISK;

    GemmParams g{};
    g.W = reinterpret_cast<const uint32_t *>(Fp);
    g.A = reinterpret_cast<const uint32_t *>(in);
    g.M = F; g.N = (int)N; g.Kd = (int)(2 * S);
    set_coefficients(g, wbits, wfmt, abits, afmt, Kl);
    g.C = nullptr; g.ldc = 0;
    g.thr = thr; g.obits = obits; g.T = (1 << obits) - 1;
    g.Y = reinterpret_cast<uint32_t *>(Yp);
    g.Yd = (int)(2 * bs_words_per_row(F));
    g.cH = PH; g.cW = PW; g.cCd = (C + 31) / 32; g.cPix = (int)pix; g.cKW = kw;
    g.cStride = stride; g.cPad = pad; g.cOW = OW; g.cOHW = OH * OW; g.cB = B; g.cKused = (int)(Kl / 32);
    g.cVec = (g.cCd % 4 == 0 && g.cPix % 4 == 0) ? 1 : 0;
    g.pK = pool_k > 0 ? pool_k : 0; g.pS = pool_stride; g.pH = H; g.pW = W;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool corr = (wfmt == BS_BIPOLAR);
    if (pool_k > 0) {
        // A kernel that covers the whole pooled map is a fully connected layer on the flattened map: with few images
        // the weights are streamed once by the few-column kernel, whose activation fill does the pooling.
        if (N <= kGemvMaxCols && OH == 1 && OW == 1 && pad == 0 && kh == PH && kw == PW) {
            const int nc = N == 1 ? 1 : (N == 2 ? 2 : 4);
            if ((size_t)abits * nc * (g.Kd >> 2) * 16 <= kGemvMaxLds) {
                finish_params(g);
                return launch_gemv(g, wbits, abits, true, false, st);
            }
        }
        return dispatch_wb(g, wbits, abits, true, corr, true, false, st);
    }
    // Engine (Sec. 4.2): the layer is the product F x Kl x N; the matrix-core kernel gathers the lowered columns itself.
    if (engine != BS_ENGINE_BITSERIAL) {
        const bs_engine e = engine == BS_ENGINE_AUTO ? bs_choose_engine(wbits, wfmt, abits, afmt, F, N, Kl) : engine;
        if (e != BS_ENGINE_BITSERIAL) {
            PlanesGemm q{};
            q.W = g.W; q.A = g.A; q.wbits = wbits; q.abits = abits; q.wfmt = wfmt; q.afmt = afmt;
            q.M = g.M; q.N = g.N; q.K = Kl; q.Kd = g.Kd;
            q.thr = thr; q.obits = obits; q.Y = g.Y; q.Yd = g.Yd;
            q.conv = 1;
            q.cH = H; q.cW = W; q.cCd = g.cCd; q.cPix = g.cPix; q.cKW = kw; q.cStride = stride; q.cPad = pad;
            q.cOW = OW; q.cOHW = OH * OW; q.cB = B; q.cKused = g.cKused;
            return launch_planes_mfma(q, e == BS_ENGINE_DENSE_FP4, true, st);
        }
    }
    return dispatch_wb(g, wbits, abits, true, corr, true, false, st);
}

}  // namespace

extern "C" bs_status bs_conv_threshold_batch_on(bs_engine engine, const uint64_t *in, int abits, bs_format afmt, int B, int H,
                                                int W, int C, const uint64_t *Fp, int wbits, bs_format wfmt, int F, int kh,
                                                int kw, int stride, int pad, const int32_t *thr, int obits, uint64_t *Yp,
                                                void *stream)
{
    return conv_common(engine, in, abits, afmt, B, H, W, C, 0, 0, Fp, wbits, wfmt, F, kh, kw, stride, pad, thr, obits, Yp, stream);
}

extern "C" bs_status bs_pool_conv_threshold_batch(const uint64_t *in, int abits, int B, int H, int W, int C, int pool_k,
                                                  int pool_stride, const uint64_t *Fp, int wbits, bs_format wfmt, int F,
                                                  int kh, int kw, int stride, int pad, const int32_t *thr, int obits,
                                                  uint64_t *Yp, void *stream)
{
    if (pool_k <= 0) return BS_ERR_INVALID_ARG;
    return conv_common(BS_ENGINE_BITSERIAL, in, abits, BS_UNSIGNED, B, H, W, C, pool_k, pool_stride, Fp, wbits, wfmt, F, kh, kw,
                       stride, pad, thr, obits, Yp, stream);
}

extern "C" bs_status bs_conv_threshold_batch(const uint64_t *in, int abits, bs_format afmt, int B, int H, int W, int C,
                                             const uint64_t *Fp, int wbits, bs_format wfmt, int F, int kh, int kw,
                                             int stride, int pad, const int32_t *thr, int obits, uint64_t *Yp,
                                             void *stream)
{
    return bs_conv_threshold_batch_on(BS_ENGINE_AUTO, in, abits, afmt, B, H, W, C, Fp, wbits, wfmt, F, kh, kw, stride, pad, thr,
                                      obits, Yp, stream);
}

extern "C" bs_status bs_conv_threshold(const uint64_t *in, int abits, bs_format afmt, int H, int W, int C,
                                       const uint64_t *Fp, int wbits, bs_format wfmt, int F, int kh, int kw,
                                       int stride, int pad, const int32_t *thr, int obits, uint64_t *Yp, void *stream)
{
    return bs_conv_threshold_batch(in, abits, afmt, 1, H, W, C, Fp, wbits, wfmt, F, kh, kw, stride, pad, thr, obits, Yp,
                                   stream);
}

extern "C" bs_status bs_gemm_topbits(const uint64_t *Wp, int wbits, bs_format wfmt, const uint64_t *Ap, int abits,
                                     bs_format afmt, int64_t M, int64_t N, int64_t K, int min_shift, int32_t *C,
                                     int64_t ldc, void *stream)
{
    if (min_shift < 0 || min_shift > wbits + abits - 2) return BS_ERR_INVALID_ARG;
    return gemm_common(BS_ENGINE_BITSERIAL, Wp, wbits, wfmt, Ap, abits, afmt, M, N, K, C, ldc, nullptr, 0, nullptr, false, stream,
                       min_shift);
}
