// Channel-interleaved lowering on packed data (Sec. 3.2 of the paper): the feature map
// is kept as one bit plane per activation bit, each pixel holding that bit of all its
// channels padded to a word, so the sliding-window copy of im2col moves whole words and
// needs no masking or shifting.  The word here is 32 bits (the register width of the
// chip): a pixel contributes ceil(C/32) words to every lowered column it appears in.
//
// One thread writes one 32-bit word of the lowered matrix; consecutive lanes write
// consecutive words of a column, so stores coalesce and the reads are short contiguous
// runs (one pixel) that hit in cache across neighbouring columns.
#include "bs_common.h"

namespace {

struct LowerParams {
    const uint32_t *in;
    uint32_t *out;
    int H, W, Cd;      // Cd = 32-bit words copied per pixel
    int pix_d;         // 32-bit words between pixels in `in`
    int kh, kw, stride, pad;
    int OH, OW;
    int Kd_used;       // kh * kw * Cd
    int out_d;         // 32-bit words per lowered column (row stride of `out`)
    int abits;
};

__global__ void __launch_bounds__(256) im2col_kernel(const LowerParams p)
{
    const int q = blockIdx.x * 256 + threadIdx.x;     // word within the lowered column
    const int col = blockIdx.y;                       // output pixel
    const int plane = blockIdx.z;
    if (q >= p.out_d) return;
    uint32_t v = 0;
    if (q < p.Kd_used) {
        const int tap = q / p.Cd, cd = q - tap * p.Cd;
        const int r = tap / p.kw, s = tap - r * p.kw;
        const int oh = col / p.OW, ow = col - oh * p.OW;
        const int ih = oh * p.stride + r - p.pad, iw = ow * p.stride + s - p.pad;
        if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
            v = p.in[((size_t)plane * p.H * p.W + (size_t)ih * p.W + iw) * p.pix_d + cd];
    }
    p.out[((size_t)plane * p.OH * p.OW + col) * p.out_d + q] = v;
}

}  // namespace

extern "C" int64_t bs_lowered_depth(int64_t C, int64_t kh, int64_t kw)
{
    if (C <= 0 || kh <= 0 || kw <= 0) return 0;
    return kh * kw * 32 * ((C + 31) / 32);
}

extern "C" bs_status bs_im2col_interleaved(const uint64_t *in, int abits, int H, int W, int C, int kh, int kw,
                                           int stride, int pad, uint64_t *out, void *stream)
{
    if (!in || !out || abits < 1 || H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0)
        return BS_ERR_INVALID_ARG;
    if (abits > bs::kMaxBits) return BS_ERR_UNSUPPORTED;
    if (H + 2 * pad < kh || W + 2 * pad < kw) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(in, 16) || !bs::aligned(out, 16)) return BS_ERR_ALIGNMENT;
    LowerParams p;
    p.in = reinterpret_cast<const uint32_t *>(in);
    p.out = reinterpret_cast<uint32_t *>(out);
    p.H = H; p.W = W; p.Cd = (C + 31) / 32;
    p.pix_d = (int)(2 * bs_words_per_row(C));
    p.kh = kh; p.kw = kw; p.stride = stride; p.pad = pad;
    p.OH = (H + 2 * pad - kh) / stride + 1;
    p.OW = (W + 2 * pad - kw) / stride + 1;
    const int64_t Kl = bs_lowered_depth(C, kh, kw);
    const int64_t out_d = 2 * bs_words_per_row(Kl);
    const int64_t ncol = (int64_t)p.OH * p.OW;
    if (out_d * ncol * abits >= (int64_t(1) << 31) || ncol > 65535 * 32768LL) return BS_ERR_OVERFLOW_RISK;
    p.Kd_used = (int)(Kl / 32);
    p.out_d = (int)out_d;
    p.abits = abits;
    if (ncol > 65535) return BS_ERR_UNSUPPORTED;
    dim3 grid((unsigned)((out_d + 255) / 256), (unsigned)ncol, (unsigned)abits);
    im2col_kernel<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(p);
    return bs::after_launch();
}
