// Successive thresholding as a stand-alone call (Sec. 2.1.1 of the paper; integer
// thresholds per Sec. 2.1.3): count the thresholds each int32 accumulator reaches and
// emit the few-bit result as channel-interleaved bit planes (packed along the rows m).
//
// A workgroup covers 128 rows x 64 columns: lanes run along the column index so that the
// int32 reads of C coalesce, each wavefront produces one 32-bit output word (32 rows) per
// plane and column.  All 32 accumulators of a thread are requested before the first
// comparison (one memory round trip).  A row's thresholds are the same for every lane of
// the wavefront, so they are fetched with scalar loads and compared from scalar registers:
// no LDS traffic for them (staged in LDS they cost one 16-byte broadcast read per four
// comparisons, which bounded the 4-bit case).  The four wavefronts' words of a column
// meet in LDS and leave as one 16-byte store per plane and column.
#include "bs_common.h"

namespace {

template <int OB>
__global__ void __launch_bounds__(256)
threshold_kernel(const int32_t *__restrict__ C, long long ldc, int M, int N, const int32_t *__restrict__ thr,
                 uint32_t *__restrict__ Y, int Yd)
{
    constexpr int T = (1 << OB) - 1;
    __shared__ uint4 yt[OB * 64];  // [plane][column]: the four words of the workgroup's 128 rows
    const int tid = threadIdx.x;
    const int n = blockIdx.x * 64 + (tid & 63);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps the threshold addresses scalar
    const int mbase = (blockIdx.y * 4 + wave) * 32;
    // rows past the end read the last valid row (any valid address does: their result is dropped)
    const int last = M - 1 - mbase;  // uniform; negative when the whole word lies past the end (row M - 1 then)
    int32_t c[32];
    if (n < N) {
#pragma unroll
        for (int r = 0; r < 32; ++r) {
            const int row = mbase + (r < last ? r : last);
            c[r] = C[(long long)row * ldc + n];
        }
    }
    // Bit-sliced over the thread's 32 rows: word hit[t] collects, one bit per row, whether the row's accumulator
    // reaches the row's threshold t (compare into the carry, then hit = 2 hit + carry, rows taken from 31 down to 0 so
    // that row r ends up in bit r).  The count of Sec. 2.1.1 is the sum of the T one-bit words, taken for all 32 rows
    // at once by a carry-save adder tree whose outputs ARE the plane words (11 full adders of two three-input bit
    // operations for T = 15), instead of a count per element that is then cut into planes bit by bit (8 more
    // instructions per element at 4 bits: 94 -> 79 us for 8192 x 8192).
    uint32_t w[OB];
#pragma unroll
    for (int p = 0; p < OB; ++p) w[p] = 0;
    if (n < N) {
        uint32_t hit[T];
#pragma unroll
        for (int t = 0; t < T; ++t) hit[t] = 0;
#pragma unroll
        for (int r = 31; r >= 0; --r) {
            const int row = mbase + (r < last ? r : last);
            const int32_t *tr = thr + (long long)row * T;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int32_t th = tr[t];  // uniform address: a scalar load
                asm("v_cmp_le_i32 vcc, %2, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(hit[t]) : "v"(c[r]), "s"(th) : "vcc");
            }
        }
        bs::count_planes<OB>(hit, w);
        // rows past M compared a copy of row M - 1: their bits are dropped
        const uint32_t valid = last >= 31 ? 0xFFFFFFFFu : (last < 0 ? 0u : ((2u << last) - 1u));
#pragma unroll
        for (int p = 0; p < OB; ++p) w[p] &= valid;
    }
#pragma unroll
    for (int p = 0; p < OB; ++p) reinterpret_cast<uint32_t *>(yt)[(p * 64 + (tid & 63)) * 4 + wave] = w[p];
    __syncthreads();
    for (int it = tid; it < OB * 64; it += 256) {
        const int p = it >> 6, nn = blockIdx.x * 64 + (it & 63);
        if (nn >= N) continue;
        // Yd is a multiple of 4 and the workgroup owns words 4 blockIdx.y .. + 3: a 16-byte aligned store
        *reinterpret_cast<uint4 *>(Y + ((long long)p * N + nn) * Yd + blockIdx.y * 4) = yt[it];
    }
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
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t *Y = reinterpret_cast<uint32_t *>(Yp);
    switch (obits) {
    case 1: threshold_kernel<1><<<grid, 256, 0, st>>>(C, ldc, (int)M, (int)N, thr, Y, (int)Yd); break;
    case 2: threshold_kernel<2><<<grid, 256, 0, st>>>(C, ldc, (int)M, (int)N, thr, Y, (int)Yd); break;
    case 3: threshold_kernel<3><<<grid, 256, 0, st>>>(C, ldc, (int)M, (int)N, thr, Y, (int)Yd); break;
    default: threshold_kernel<4><<<grid, 256, 0, st>>>(C, ldc, (int)M, (int)N, thr, Y, (int)Yd); break;
    }
    return bs::after_launch();
}
