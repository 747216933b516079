// Status strings and version of libbsgemm.
#include "bs_common.h"

extern "C" const char *bs_status_string(bs_status s)
{
    switch (s) {
    case BS_OK: return "ok";
    case BS_ERR_INVALID_ARG: return "invalid argument";
    case BS_ERR_UNSUPPORTED: return "unsupported configuration";
    case BS_ERR_ALIGNMENT: return "misaligned pointer or leading dimension";
    case BS_ERR_OVERFLOW_RISK: return "int32 accumulator or 32-bit index could overflow";
    case BS_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

extern "C" int bs_version(void) { return 100; }

// Per-layer engine choice (Sec. 4.1.1 / 4.2): the fastest of the engines under a time model whose
// constants were fitted to measurements over M, N in 256..4096, K in {1024, 4096} and W1A1, W1A2,
// W2A2, W4A4 on MI355X (fused 2^abits-level epilogue, activation unpack counted for the dense
// engines; non-negative least squares on the relative error, which stays within -18 / +29 % bit-serial,
// -33 / +12 % int8, -17 / +11 % fp4; over the measured cases the choice costs 0.4 % on average and 17 % at
// worst against always picking the fastest).  Microseconds.
// The dense engines as the library runs them on packed planes: 4-bit floating-point codes for operands of at most two
// bits while the fp32 accumulation stays exact, int8 otherwise; both count depth indices in 32 bits.
static bool fp4_usable(int wbits, bs_format wfmt, int abits, bs_format afmt, int64_t K)
{
    (void)wfmt; (void)afmt;  // the kernel multiplies unsigned codes, whatever the format
    return wbits <= 2 && abits <= 2 && K * ((int64_t(1) << wbits) - 1) * ((int64_t(1) << abits) - 1) < (int64_t(1) << 24);
}

extern "C" bs_engine bs_choose_engine(int wbits, bs_format wfmt, int abits, bs_format afmt, int64_t M, int64_t N, int64_t K)
{
    if (wbits < 1 || wbits > 4 || abits < 1 || abits > 4 || M <= 0 || N <= 0 || K <= 0) return BS_ENGINE_BITSERIAL;
    if ((wfmt == BS_BIPOLAR && wbits != 1) || (afmt == BS_BIPOLAR && abits != 1)) return BS_ENGINE_BITSERIAL;
    if (K >= (int64_t(1) << 30)) return BS_ENGINE_BITSERIAL;  // beyond the dense engines' depth range
    if (N <= 4) return BS_ENGINE_BITSERIAL;  // weights streamed once: wbits/8 byte per weight beats a byte or half a byte
    const double pairs = (double)wbits * abits, kk = (double)K / 1024.0;
    const double mnk2 = 2.0 * (double)M * (double)N * (double)K, mn = (double)M * (double)N;
    // 5..16 columns: the bit-serial call takes the faster of the streaming kernel in groups of four columns and
    // the tiled kernel with 32 x 8 tiles (the same two models decide inside bs_gemm)
    double t_bitserial = 4.8 + 0.21 * kk * pairs + mnk2 * pairs / 1.13e9;
    if (N <= 16) {
        const double groups = (double)((N + 3) / 4) * (double)M / 4096.0;
        const double t_stream = 3.88 + groups * (0.69 + 0.2 * pairs + 0.031 * pairs * kk);
        const double blocks = (double)((M + 31) / 32) * (double)((N + 7) / 8);
        const double rounds = 1.0 + (blocks > 256.0 ? (blocks - 256.0) / 900.0 : 0.0);
        const double t_tiled = 3.64 + rounds * pairs * (0.253 * kk + 0.21);
        t_bitserial = t_stream < t_tiled ? t_stream : t_tiled;
    }
    if (fp4_usable(wbits, wfmt, abits, afmt, K)) {
        const double t_fp4 = 4.2 + 2.2 * kk + 1.1 * abits + mnk2 / 6.63e9 + mn / 3.92e6;
        return t_fp4 < t_bitserial ? BS_ENGINE_DENSE_FP4 : BS_ENGINE_BITSERIAL;  // measured 1.1 - 1.5 x faster than int8 everywhere
    }
    const double t_int8 = 3.2 + 4.3 * kk + 1.8 * abits + mnk2 / 4.07e9 + mn / 2.18e6;
    return t_int8 < t_bitserial ? BS_ENGINE_DENSE_I8 : BS_ENGINE_BITSERIAL;
}
