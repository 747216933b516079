// Host side of the few-column kernels (bs_gemv_kernel.h): when they apply, and dispatch on the number of weight planes.
#include "bs_gemv_kernel.h"

namespace bs {
extern template bs_status launch_gemv_wb<1>(const GemmParams &, int, bool, bool, hipStream_t);
extern template bs_status launch_gemv_wb<2>(const GemmParams &, int, bool, bool, hipStream_t);
extern template bs_status launch_gemv_wb<3>(const GemmParams &, int, bool, bool, hipStream_t);
extern template bs_status launch_gemv_wb<4>(const GemmParams &, int, bool, bool, hipStream_t);

bool gemv_applicable(const GemmParams &g, int wbits, int abits, bool a_bipolar, bool w_bipolar)
{
    // bipolar activations are handled in the XOR form only (both operands bipolar)
    if (g.N > kGemvMaxGroupedCols || (a_bipolar && !w_bipolar)) return false;
    const int nc = g.N == 1 ? 1 : (g.N == 2 ? 2 : 4);
    if ((size_t)abits * nc * (g.Kd >> 2) * 16 > kGemvMaxLds) return false;
    if (g.N <= kGemvMaxCols) return true;  // one group: every weight word is read once
    // 5..16 columns: groups of four stream the weights again and pay a fixed cost per row and group, while the
    // tiled kernel (32 x 8 tiles, up to 256 workgroups at once without slowing down) pays per depth stage.  Time
    // models in microseconds fitted to W1A2, W2A2, W4A4 at M = 1024..16384, depth 256..9216, N = 5..16 (180
    // shapes: the choice is within 0.24 % of the faster kernel on average, 8 % at worst; always taking this
    // kernel would cost 72 % on average, 5x at 16384 rows); p = plane pairs, k = depth / 1024.
    const double p = (double)wbits * abits, k = (double)g.Kd / 32.0;
    const double groups = (double)((g.N + 3) / 4) * (double)g.M / 4096.0;
    const double t_gemv = 3.88 + groups * (0.69 + 0.2 * p + 0.031 * p * k);
    const double blocks = (double)((g.M + 31) / 32) * (double)((g.N + 7) / 8);
    const double rounds = 1.0 + (blocks > 256.0 ? (blocks - 256.0) / 900.0 : 0.0);
    const double t_tiled = 3.64 + rounds * p * (0.253 * k + 0.21);
    return t_gemv <= t_tiled;
}

bs_status launch_gemv(const GemmParams &g, int wbits, int abits, bool fuse, bool xr, hipStream_t st)
{
    switch (wbits) {
    case 1: return launch_gemv_wb<1>(g, abits, fuse, xr, st);
    case 2: return launch_gemv_wb<2>(g, abits, fuse, xr, st);
    case 3: return launch_gemv_wb<3>(g, abits, fuse, xr, st);
    default: return launch_gemv_wb<4>(g, abits, fuse, xr, st);
    }
}

}  // namespace bs
