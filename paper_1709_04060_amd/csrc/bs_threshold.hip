// Successive thresholding as a stand-alone call (Sec. 2.1.1 of the paper; integer
// thresholds per Sec. 2.1.3): count the thresholds each int32 accumulator reaches and
// emit the few-bit result as channel-interleaved bit planes (packed along the rows m).
//
// One thread produces one 32-bit output word per plane: 32 consecutive rows of one
// column.  Lanes run along the column index so that the int32 reads of C coalesce; the
// 32 rows of a word are uniform across the wavefront, so their thresholds are read
// once per wavefront through the scalar path.
#include "bs_common.h"

namespace {

__global__ void __launch_bounds__(256)
threshold_kernel(const int32_t *__restrict__ C, long long ldc, int M, int N, const int32_t *__restrict__ thr, int T,
                 int obits, uint32_t *__restrict__ Y, int Yd)
{
    const int n = blockIdx.x * 64 + (threadIdx.x & 63);
    const int wi = blockIdx.y * 4 + (threadIdx.x >> 6);   // output dword index within the column
    if (wi >= Yd || n >= N) return;
    uint32_t w[bs::kMaxBits] = {0, 0, 0, 0};
    const int mbase = wi * 32;
    for (int r = 0; r < 32; ++r) {
        const int m = mbase + r;
        if (m >= M) break;
        const int32_t c = C[(long long)m * ldc + n];
        const int32_t *th = thr + (long long)m * T;
        uint32_t y = 0;
        for (int t = 0; t < T; ++t) y += (c >= th[t]) ? 1u : 0u;
#pragma unroll
        for (int p = 0; p < bs::kMaxBits; ++p) w[p] |= ((y >> p) & 1u) << r;
    }
    for (int p = 0; p < obits; ++p) Y[((long long)p * N + n) * Yd + wi] = w[p];
}

}  // namespace

extern "C" bs_status bs_threshold_activate(const int32_t *C, int64_t ldc, int64_t M, int64_t N, const int32_t *thr,
                                           int obits, uint64_t *Yp, void *stream)
{
    if (!C || !thr || !Yp || M <= 0 || N <= 0 || ldc < N || obits < 1) return BS_ERR_INVALID_ARG;
    if (obits > bs::kMaxBits) return BS_ERR_UNSUPPORTED;
    if (!bs::aligned(C, 4) || !bs::aligned(thr, 4) || !bs::aligned(Yp, 16)) return BS_ERR_ALIGNMENT;
    const int64_t Yd = 2 * bs_words_per_row(M);
    if (M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31) || obits * N * Yd >= (int64_t(1) << 31))
        return BS_ERR_OVERFLOW_RISK;
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)((Yd + 3) / 4));
    if (grid.y > 65535) return BS_ERR_UNSUPPORTED;
    threshold_kernel<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(
        C, ldc, (int)M, (int)N, thr, (1 << obits) - 1, obits, reinterpret_cast<uint32_t *>(Yp), (int)Yd);
    return bs::after_launch();
}
