// Max pooling on packed, channel-interleaved bit planes.  The paper keeps pooling outside
// its hot path (Sec. 4.2, run as a float layer); thresholding is monotone, so pooling the
// thresholded codes is exact, and doing it on the packed planes lets the quantized
// layers of Table 2 run as one chain without unpacking.
//
// The maximum of two b-bit numbers held bit-sliced (one word per bit position, 32
// channels per word) is a most-significant-bit-first comparison in pure bitwise logic.
// One thread owns one 32-bit channel word of one output pixel, for all planes.
#include "bs_common.h"

namespace {

struct PoolParams {
    const uint32_t *in;
    uint32_t *out;
    int bits, B, H, W, pix_d, k, stride, OH, OW;
};

// KW > 0: window size known at compile time, so all taps are loaded before the first
// comparison (one memory round trip instead of one per tap).  KW == 0: any window size.
template <int KW>
__global__ void __launch_bounds__(256) maxpool_kernel(const PoolParams p)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int total = p.B * p.OH * p.OW * p.pix_d;
    if (idx >= total) return;
    const int cd = idx % p.pix_d, bpix = idx / p.pix_d;
    const int img = bpix / (p.OH * p.OW), opix = bpix - img * (p.OH * p.OW);
    const int oh = opix / p.OW, ow = opix - oh * p.OW;
    const size_t in_plane = (size_t)p.B * p.H * p.W * p.pix_d, out_plane = (size_t)total;
    const size_t in_img = (size_t)img * p.H * p.W * p.pix_d;

    uint32_t best[bs::kMaxBits] = {0, 0, 0, 0};  // codes are unsigned: zero is the identity of max
    // per channel (bit lane): gt = v > best, decided at the highest differing plane
    auto take_max = [&](const uint32_t (&v)[bs::kMaxBits]) {
        uint32_t gt = 0, eq = 0xFFFFFFFFu;
#pragma unroll
        for (int b = bs::kMaxBits - 1; b >= 0; --b) {
            gt |= eq & v[b] & ~best[b];
            eq &= ~(v[b] ^ best[b]);
        }
#pragma unroll
        for (int b = 0; b < bs::kMaxBits; ++b) best[b] = (gt & v[b]) | (~gt & best[b]);
    };
    if constexpr (KW > 0) {
        uint32_t v[KW * KW][bs::kMaxBits];
#pragma unroll
        for (int r = 0; r < KW; ++r)
#pragma unroll
            for (int s = 0; s < KW; ++s) {
                const size_t at = in_img + ((size_t)(oh * p.stride + r) * p.W + (ow * p.stride + s)) * p.pix_d + cd;
#pragma unroll
                for (int b = 0; b < bs::kMaxBits; ++b) v[r * KW + s][b] = b < p.bits ? p.in[b * in_plane + at] : 0u;
            }
#pragma unroll
        for (int t = 0; t < KW * KW; ++t) take_max(v[t]);
    } else {
        for (int r = 0; r < p.k; ++r)
            for (int s = 0; s < p.k; ++s) {
                const size_t at = in_img + ((size_t)(oh * p.stride + r) * p.W + (ow * p.stride + s)) * p.pix_d + cd;
                uint32_t v[bs::kMaxBits] = {0, 0, 0, 0};
                for (int b = 0; b < p.bits; ++b) v[b] = p.in[b * in_plane + at];
                take_max(v);
            }
    }
    for (int b = 0; b < p.bits; ++b) p.out[b * out_plane + idx] = best[b];
}

}  // namespace

extern "C" bs_status bs_maxpool_packed_batch(const uint64_t *in, int bits, int B, int H, int W, int C, int k,
                                             int stride, uint64_t *out, void *stream)
{
    if (!in || !out || bits < 1 || B <= 0 || H <= 0 || W <= 0 || C <= 0 || k <= 0 || stride <= 0 || k > H || k > W)
        return BS_ERR_INVALID_ARG;
    if (bits > bs::kMaxBits) return BS_ERR_UNSUPPORTED;
    if (!bs::aligned(in, 16) || !bs::aligned(out, 16)) return BS_ERR_ALIGNMENT;
    PoolParams p;
    p.in = reinterpret_cast<const uint32_t *>(in);
    p.out = reinterpret_cast<uint32_t *>(out);
    p.bits = bits; p.B = B; p.H = H; p.W = W; p.k = k; p.stride = stride;
    p.pix_d = (int)(2 * bs_words_per_row(C));
    p.OH = (H - k) / stride + 1;
    p.OW = (W - k) / stride + 1;
    const int64_t total = (int64_t)B * p.OH * p.OW * p.pix_d;
    if ((int64_t)bits * B * H * W * p.pix_d >= (int64_t(1) << 31)) return BS_ERR_OVERFLOW_RISK;
    const dim3 grid((unsigned)((total + 255) / 256));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (k == 2) maxpool_kernel<2><<<grid, 256, 0, st>>>(p);
    else if (k == 3) maxpool_kernel<3><<<grid, 256, 0, st>>>(p);
    else maxpool_kernel<0><<<grid, 256, 0, st>>>(p);
    return bs::after_launch();
}

extern "C" bs_status bs_maxpool_packed(const uint64_t *in, int bits, int H, int W, int C, int k, int stride,
                                       uint64_t *out, void *stream)
{
    return bs_maxpool_packed_batch(in, bits, 1, H, W, C, k, stride, out, stream);
}
