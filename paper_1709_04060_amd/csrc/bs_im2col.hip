// Channel-interleaved lowering on packed data (Sec. 3.2 of the paper): the feature map
// is kept as one bit plane per activation bit, each pixel holding that bit of all its
// channels padded to a word, so the sliding-window copy of im2col moves whole words and
// needs no masking or shifting.  The word here is 32 bits (the register width of the
// chip): a pixel contributes ceil(C/32) words to every lowered column it appears in.
//
// One thread writes one 16-byte chunk (four words) of the lowered matrix; consecutive
// lanes write consecutive chunks of a column and then of the next column, so stores
// coalesce, and the reads are short contiguous runs (one pixel) that hit in cache across
// neighbouring columns.  A batch of images puts its columns side by side (column = image *
// OH * OW + output pixel): the grid's second dimension walks (plane, image), so the index
// arithmetic (four 32-bit divisions per thread) stays inside one image.  When a pixel's run
// is a multiple of four words (channels a multiple of 128) a chunk lies inside one tap and
// is one 16-byte load; otherwise its four words are gathered one by one.
#include "bs_common.h"

namespace {

struct LowerParams {
    const uint32_t *in;
    uint32_t *out;
    int H, W, Cd;      // Cd = 32-bit words copied per pixel
    int pix_d;         // 32-bit words between pixels in `in`
    int kw, stride, pad;
    int OW;
    int Kd_used;       // kh * kw * Cd
    int nch;           // 16-byte chunks per lowered column (row stride of `out` / 4)
    int img_chunks;    // OH * OW * nch: chunks of one image's lowered matrix in one plane
    int maps;          // abits * B feature maps
    int vec;           // Cd and pix_d are multiples of 4
};

__global__ void __launch_bounds__(256) im2col_kernel(const LowerParams p)
{
    const unsigned idx = blockIdx.x * 256u + threadIdx.x;   // chunk within one map's lowered matrix
    if (idx >= (unsigned)p.img_chunks) return;
    const unsigned opix = idx / (unsigned)p.nch, c4 = idx - opix * p.nch;
    const unsigned oh = opix / (unsigned)p.OW, ow = opix - oh * p.OW;
    const int ih0 = (int)oh * p.stride - p.pad, iw0 = (int)ow * p.stride - p.pad;
    const unsigned q = c4 * 4;                              // first word of the chunk within the column
    const unsigned tap = q / (unsigned)p.Cd, cd = q - tap * p.Cd;
    const unsigned r = tap / (unsigned)p.kw, s = tap - r * p.kw;
    const size_t map_d = (size_t)p.H * p.W * p.pix_d;
    for (unsigned m = blockIdx.y; m < (unsigned)p.maps; m += gridDim.y) {  // m = plane * B + image, as in the input
        const uint32_t *src = p.in + m * map_d;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (p.vec) {
            const int ih = ih0 + (int)r, iw = iw0 + (int)s;
            if (q < (unsigned)p.Kd_used && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
                v = *reinterpret_cast<const uint4 *>(src + ((size_t)ih * p.W + iw) * p.pix_d + cd);
        } else {
            unsigned rr = r, ss = s, cc = cd;
            uint32_t e[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                e[t] = 0;
                const int ih = ih0 + (int)rr, iw = iw0 + (int)ss;
                if (q + t < (unsigned)p.Kd_used && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
                    e[t] = src[((size_t)ih * p.W + iw) * p.pix_d + cc];
                if (++cc == (unsigned)p.Cd) {
                    cc = 0;
                    if (++ss == (unsigned)p.kw) { ss = 0; ++rr; }
                }
            }
            v = make_uint4(e[0], e[1], e[2], e[3]);
        }
        *reinterpret_cast<uint4 *>(p.out + ((size_t)m * p.img_chunks + idx) * 4) = v;
    }
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
    p.H = H; p.W = W; p.Cd = (C + 31) / 32;
    p.pix_d = (int)(2 * bs_words_per_row(C));
    p.kw = kw; p.stride = stride; p.pad = pad;
    const int OH = (H + 2 * pad - kh) / stride + 1;
    p.OW = (W + 2 * pad - kw) / stride + 1;
    const int64_t Kl = bs_lowered_depth(C, kh, kw);
    const int64_t out_d = 2 * bs_words_per_row(Kl);  // a multiple of 4: rows are padded to 16 bytes
    const int64_t ncol = (int64_t)B * OH * p.OW;
    const int64_t lim = int64_t(1) << 31;
    if (out_d * ncol * abits >= lim || (int64_t)abits * B * H * W * p.pix_d >= lim) return BS_ERR_OVERFLOW_RISK;
    p.Kd_used = (int)(Kl / 32);
    p.nch = (int)(out_d / 4);
    p.img_chunks = OH * p.OW * p.nch;
    p.maps = abits * B;
    p.vec = (p.Cd % 4 == 0 && p.pix_d % 4 == 0) ? 1 : 0;
    const dim3 grid((unsigned)((p.img_chunks + 255) / 256), (unsigned)(p.maps < 65535 ? p.maps : 65535));
    im2col_kernel<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(p);
    return bs::after_launch();
}

extern "C" bs_status bs_im2col_interleaved(const uint64_t *in, int abits, int H, int W, int C, int kh, int kw,
                                           int stride, int pad, uint64_t *out, void *stream)
{
    return bs_im2col_interleaved_batch(in, abits, 1, H, W, C, kh, kw, stride, pad, out, stream);
}
