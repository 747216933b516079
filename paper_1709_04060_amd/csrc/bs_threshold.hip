// Successive thresholding as a stand-alone call (Sec. 2.1.1 of the paper; integer
// thresholds per Sec. 2.1.3): count the thresholds each int32 accumulator reaches and
// emit the few-bit result as channel-interleaved bit planes (packed along the rows m).
//
// A workgroup covers 128 rows x 64 columns: lanes run along the column index so that the
// int32 reads of C coalesce, each wavefront produces one 32-bit output word (32 rows) per
// plane and column.  All 32 accumulators of a thread are requested before the first
// comparison (one memory round trip), and the thresholds of the 128 rows are staged in LDS,
// padded to 16 per row with INT_MAX (never reached) and read as 16-byte groups that every
// lane of a wavefront shares.
#include "bs_common.h"

namespace {

__global__ void __launch_bounds__(256)
threshold_kernel(const int32_t *__restrict__ C, long long ldc, int M, int N, const int32_t *__restrict__ thr, int T,
                 int obits, uint32_t *__restrict__ Y, int Yd)
{
    __shared__ int4 tl[128 * 4];  // [row of the block][4 groups of 4 thresholds]
    const int tid = threadIdx.x;
    const int n = blockIdx.x * 64 + (tid & 63);
    const int wi = blockIdx.y * 4 + (tid >> 6);       // output dword index within the column
    const int mblock = blockIdx.y * 128;
    for (int it = tid; it < 128 * 16; it += 256) {
        const int r = it >> 4, t = it & 15;
        reinterpret_cast<int32_t *>(tl)[it] =
            (mblock + r < M && t < T) ? thr[(long long)(mblock + r) * T + t] : 0x7fffffff;
    }
    const int mbase = wi * 32;
    int32_t c[32];
    if (wi < Yd && n < N) {
#pragma unroll
        for (int r = 0; r < 32; ++r) c[r] = (mbase + r < M) ? C[(long long)(mbase + r) * ldc + n] : 0;
    }
    __syncthreads();
    if (wi >= Yd || n >= N) return;
    const int nq = (T + 3) >> 2;
    uint32_t w[bs::kMaxBits] = {0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        uint32_t y = 0;
        for (int q = 0; q < nq; ++q) {
            const int4 th = tl[((tid >> 6) * 32 + r) * 4 + q];
            y += (uint32_t)(c[r] >= th.x) + (uint32_t)(c[r] >= th.y) + (uint32_t)(c[r] >= th.z) + (uint32_t)(c[r] >= th.w);
        }
        if (mbase + r >= M) y = 0;
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
