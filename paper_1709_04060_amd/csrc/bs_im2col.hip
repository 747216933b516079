// Channel-interleaved lowering on packed data (Sec. 3.2 of the paper): the feature map
// is kept as one bit plane per activation bit, each pixel holding that bit of all its
// channels padded to a word, so the sliding-window copy of im2col moves whole words and
// needs no masking or shifting.  The word here is 32 bits (the register width of the
// chip): a pixel contributes ceil(C/32) words to every lowered column it appears in.
//
// One thread writes one 32-bit word of the lowered matrix; consecutive lanes write
// consecutive words of a column, so stores coalesce and the reads are short contiguous
// runs (one pixel) that hit in cache across neighbouring columns.  A batch of images puts
// its columns side by side (column = image * OH * OW + output pixel).
#include "bs_common.h"

namespace {

struct LowerParams {
    const uint32_t *in;
    uint32_t *out;
    int B, H, W, Cd;   // Cd = 32-bit words copied per pixel
    int pix_d;         // 32-bit words between pixels in `in`
    int kh, kw, stride, pad;
    int OH, OW;
    int Kd_used;       // kh * kw * Cd
    int out_d;         // 32-bit words per lowered column (row stride of `out`)
    long long total;   // abits * B * OH * OW * out_d words to write
};

__global__ void __launch_bounds__(256) im2col_kernel(const LowerParams p)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= p.total) return;
    const int q = (int)(idx % p.out_d);               // word within the lowered column
    const long long pc = idx / p.out_d;               // (plane, image, output pixel)
    const int ohw = p.OH * p.OW;
    const int opix = (int)(pc % ohw);
    const long long pb = pc / ohw;                     // plane * B + image: the same product indexes the input maps
    uint32_t v = 0;
    if (q < p.Kd_used) {
        const int tap = q / p.Cd, cd = q - tap * p.Cd;
        const int r = tap / p.kw, s = tap - r * p.kw;
        const int oh = opix / p.OW, ow = opix - oh * p.OW;
        const int ih = oh * p.stride + r - p.pad, iw = ow * p.stride + s - p.pad;
        if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
            v = p.in[((size_t)pb * p.H * p.W + (size_t)ih * p.W + iw) * p.pix_d + cd];
    }
    p.out[idx] = v;
}

}  // namespace

extern "C" int64_t bs_lowered_depth(int64_t C, int64_t kh, int64_t kw)
{
    if (C <= 0 || kh <= 0 || kw <= 0) return 0;
    return kh * kw * 32 * ((C + 31) / 32);
}

extern "C" bs_status bs_im2col_interleaved_batch(const uint64_t *in, int abits, int B, int H, int W, int C, int kh,
                                                 int kw, int stride, int pad, uint64_t *out, void *stream)
{
    if (!in || !out || abits < 1 || B <= 0 || H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0)
        return BS_ERR_INVALID_ARG;
    if (abits > bs::kMaxBits) return BS_ERR_UNSUPPORTED;
    if (H + 2 * pad < kh || W + 2 * pad < kw) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(in, 16) || !bs::aligned(out, 16)) return BS_ERR_ALIGNMENT;
    LowerParams p;
    p.in = reinterpret_cast<const uint32_t *>(in);
    p.out = reinterpret_cast<uint32_t *>(out);
    p.B = B; p.H = H; p.W = W; p.Cd = (C + 31) / 32;
    p.pix_d = (int)(2 * bs_words_per_row(C));
    p.kh = kh; p.kw = kw; p.stride = stride; p.pad = pad;
    p.OH = (H + 2 * pad - kh) / stride + 1;
    p.OW = (W + 2 * pad - kw) / stride + 1;
    const int64_t Kl = bs_lowered_depth(C, kh, kw);
    const int64_t out_d = 2 * bs_words_per_row(Kl);
    const int64_t ncol = (int64_t)B * p.OH * p.OW;
    const int64_t lim = int64_t(1) << 31;
    if (out_d * ncol * abits >= lim || (int64_t)abits * B * H * W * p.pix_d >= lim) return BS_ERR_OVERFLOW_RISK;
    p.Kd_used = (int)(Kl / 32);
    p.out_d = (int)out_d;
    p.total = out_d * ncol * abits;
    im2col_kernel<<<dim3((unsigned)((p.total + 255) / 256)), 256, 0, static_cast<hipStream_t>(stream)>>>(p);
    return bs::after_launch();
}

extern "C" bs_status bs_im2col_interleaved(const uint64_t *in, int abits, int H, int W, int C, int kh, int kw,
                                           int stride, int pad, uint64_t *out, void *stream)
{
    return bs_im2col_interleaved_batch(in, abits, 1, H, W, C, kh, kw, stride, pad, out, stream);
}
