// Bit-plane packing (Sec. 3.1 of the paper: plane i is the binary matrix of bit i of
// every element; Alg. 1: depth packed into machine words).
//
// Two kernels, both HBM-streaming:
//  * pack_rows:  source is depth-contiguous (weights, M x K).  A wavefront reads 64
//    consecutive depth elements of one row, one per lane, and a 64-lane ballot of bit
//    p IS the packed word of plane p.
//  * pack_cols:  source is depth-strided (activations stored K x N); lanes run along
//    the contiguous N axis so loads coalesce, and each lane assembles the words of its
//    own column in registers (the transposition costs no cross-lane traffic).
#include "bs_common.h"

namespace {

template <typename T>
__device__ __forceinline__ uint32_t encode(T v, int bits, int bipolar)
{
    const int x = static_cast<int>(v);
    return bipolar ? static_cast<uint32_t>(x > 0) : (static_cast<uint32_t>(x) & ((1u << bits) - 1u));
}

// One wavefront per (row, word).  grid.x * waves_per_block wavefronts stride over
// all rows * S words.
template <typename T>
__global__ void __launch_bounds__(256)
pack_rows_kernel(const T *__restrict__ src, int64_t rows, int64_t depth, int64_t ld, int bits, int bipolar,
                 uint64_t *__restrict__ planes, int64_t S)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    const int64_t items = rows * S;
    for (int64_t it = wave; it < items; it += nwaves) {
        const int64_t r = it / S, d = it - r * S;
        const int64_t k = d * 64 + lane;
        uint32_t code = 0;
        if (k < depth) code = encode(src[r * ld + k], bits, bipolar);
        uint64_t mine = 0;
        for (int p = 0; p < bits; ++p) {
            const uint64_t word = __ballot((code >> p) & 1u);
            if (lane == p) mine = word;
        }
        if (lane < bits) planes[((int64_t)lane * rows + r) * S + d] = mine;
    }
}

// Block = 64 rows (lanes) x 4 words (wavefronts).  Element (r, k) at src[k * ld + r].
template <typename T>
__global__ void __launch_bounds__(256)
pack_cols_kernel(const T *__restrict__ src, int64_t rows, int64_t depth, int64_t ld, int bits, int bipolar,
                 uint64_t *__restrict__ planes, int64_t S)
{
    const int64_t r = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
    const int64_t d = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
    if (r >= rows || d >= S) return;
    uint64_t w[bs::kMaxBits] = {0, 0, 0, 0};
    const int64_t k0 = d * 64;
    const int kn = (int)(depth - k0 < 64 ? (depth - k0 < 0 ? 0 : depth - k0) : 64);
    for (int kk = 0; kk < kn; ++kk) {
        const uint32_t code = encode(src[(k0 + kk) * ld + r], bits, bipolar);
#pragma unroll
        for (int p = 0; p < bs::kMaxBits; ++p) w[p] |= (uint64_t)((code >> p) & 1u) << kk;
    }
    for (int p = 0; p < bits; ++p) planes[((int64_t)p * rows + r) * S + d] = w[p];
}

}  // namespace

extern "C" int64_t bs_words_per_row(int64_t depth) { return depth <= 0 ? 0 : 2 * ((depth + 127) / 128); }

extern "C" bs_status bs_pack_planes(const void *src, bs_dtype dtype, int64_t rows, int64_t depth, int64_t ld,
                                    int depth_is_strided, int bits, bs_format fmt, uint64_t *planes, void *stream)
{
    if (!src || !planes || rows <= 0 || depth <= 0) return BS_ERR_INVALID_ARG;
    if (dtype != BS_I8 && dtype != BS_I32) return BS_ERR_INVALID_ARG;
    if (bs_status s = bs::check_bits_fmt(bits, fmt)) return s;
    if (ld < (depth_is_strided ? rows : depth)) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(planes, 16)) return BS_ERR_ALIGNMENT;
    if (dtype == BS_I32 && !bs::aligned(src, 4)) return BS_ERR_ALIGNMENT;
    const int64_t S = bs_words_per_row(depth);
    if (rows * S * 2 >= (int64_t(1) << 31)) return BS_ERR_OVERFLOW_RISK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int bip = fmt == BS_BIPOLAR;
    if (!depth_is_strided) {
        const int64_t items = rows * S;
        int64_t blocks = (items + 3) / 4;
        if (blocks > 256 * 64) blocks = 256 * 64;
        if (dtype == BS_I8)
            pack_rows_kernel<int8_t><<<dim3((unsigned)blocks), 256, 0, st>>>(
                static_cast<const int8_t *>(src), rows, depth, ld, bits, bip, planes, S);
        else
            pack_rows_kernel<int32_t><<<dim3((unsigned)blocks), 256, 0, st>>>(
                static_cast<const int32_t *>(src), rows, depth, ld, bits, bip, planes, S);
    } else {
        dim3 grid((unsigned)((rows + 63) / 64), (unsigned)((S + 3) / 4));
        if (grid.y > 65535) return BS_ERR_OVERFLOW_RISK;
        if (dtype == BS_I8)
            pack_cols_kernel<int8_t><<<grid, 256, 0, st>>>(
                static_cast<const int8_t *>(src), rows, depth, ld, bits, bip, planes, S);
        else
            pack_cols_kernel<int32_t><<<grid, 256, 0, st>>>(
                static_cast<const int32_t *>(src), rows, depth, ld, bits, bip, planes, S);
    }
    return bs::after_launch();
}
