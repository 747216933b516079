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

// Per-layer engine choice (Sec. 4.1.1 / 4.2): the fastest of the engines under time models fitted to measurements on
// MI355X over M in {256, 1024, 4096}, N in {17 .. 4096}, K in {512 .. 8192} and W1A1, W1A2, W2A2, W3A3, W4A4, all from
// packed planes with the fused thresholding epilogue (375 shapes; non-negative least squares on the relative error).
// Over those shapes the choice costs 0.4 % on average and 11 % at worst against always taking the fastest engine and
// tile, where always bit-serial costs 100 % on average (20 x at worst) and always matrix cores 77 % (4.7 x).
// Microseconds.
namespace {

// The dense engines as the library runs them on packed planes: 4-bit floating-point codes for operands of at most two
// bits while the fp32 accumulation stays exact, int8 otherwise; both count depth indices in 32 bits.
bool fp4_usable(int wbits, int abits, int64_t K)
{
    return wbits <= 2 && abits <= 2 && K * ((int64_t(1) << wbits) - 1) * ((int64_t(1) << abits) - 1) < (int64_t(1) << 24);
}

// The tiled AND-popcount kernel (more than 16 columns), one model per tile the launch takes (the same steps as
// launch_planes): fixed + depth stages + stages x rounds beyond the resident workgroups + products + epilogue.
double t_bitserial_tiled(double M, double N, double K, int wbits, int abits)
{
    const long long m = (long long)M, n = (long long)N;
    const long long tiles32 = ((m + 31) / 32) * ((n + 31) / 32), tiles64 = ((m + 63) / 64) * ((n + 63) / 64);
    const double p = (double)wbits * abits, kp = K / 1024.0 * p;
    const double work = 2.0 * M * N * K * p / 1e9, epi = M * N * abits / 1e6;
    if (tiles32 <= bs::kNarrowMaxTiles32) {  // 32 x 8 tiles; a second workgroup on a compute unit slows both
        const long long blocks = ((m + 31) / 32) * ((n + 7) / 8);
        const double second = (double)((blocks + 255) / 256 - 1);
        return 3.03 + 0.206 * p + kp * (0.155 + 0.113 * second) + 1.14 * epi;
    }
    if (tiles32 <= bs::kHalfWidthMaxTiles32) return 1.98 + 0.492 * kp + 5.06 * epi;  // 32 x 16
    if (tiles64 < bs::kWideMinTiles64) return 0.38 + 0.839 * work + 3.47 * epi;      // 32 x 32, depth split
    return 1.12 + 0.612 * kp + 0.685 * work + 0.825 * epi;                           // 64 x 64
}

// The matrix-core kernel on packed planes: 256 x 256, 128 x 128 or 64 x 64 tiles (bs_planes_tile makes the same
// choice for the launch).  Time = fixed + periods x rounds x (time of a period) + epilogue, where a period (128
// depth indices as int8 codes, 256 as fp4 codes) costs more with the planes P = wbits + abits the loader has to
// request and merge, with the share `fill` of the chip's tile slots in use (the requests meet in L2), and, for the
// 128 x 128 tile, once two workgroups share a compute unit (fill > 1/2).
double t_planes(double M, double N, double K, int wbits, int abits, bool fp4)
{
    long long rounds, tiles;
    const int tile = bs_planes_tile((int64_t)M, (int64_t)N, &rounds, &tiles);
    const double nper = (double)(((int64_t)K + (fp4 ? 255 : 127)) / (fp4 ? 256 : 128));
    const double cap = tile == 256 ? 256.0 : (tile == 128 ? 512.0 : 1024.0);  // workgroups the chip holds at a time
    const double fill = ((double)tiles < cap ? (double)tiles : cap) / cap, P = wbits + abits;
    const double alone = tile == 64 ? 0.25 : 0.5;  // up to here every workgroup has a compute unit to itself
    const double shared = fill > alone ? fill - alone : 0.0;
    // fixed; per period: 1, P, fill, P fill, shared; epilogue per abits M N / 1e6
    static const double c[2][3][7] = {{{4.64, 0.613, 0.0324, 0.0000, 0.0248, 0.335, 0.316},    // int8, 64 x 64
                                       {5.69, 0.753, 0.0581, 0.0339, 0.0303, 0.285, 0.305},    // int8, 128 x 128
                                       {11.42, 1.054, 0.1341, 0.0000, 0.0738, 0.000, 0.191}},  // int8, 256 x 256
                                      {{4.48, 0.499, 0.0328, 0.0000, 0.0404, 0.320, 0.207},    // fp4, 64 x 64
                                       {5.38, 0.602, 0.0500, 0.0448, 0.0321, 0.516, 0.247},    // fp4, 128 x 128
                                       {9.29, 0.854, 0.1456, 0.0000, 0.0862, 0.000, 0.120}}}; // fp4, 256 x 256
    const double *q = c[fp4 ? 1 : 0][tile == 256 ? 2 : (tile == 128 ? 1 : 0)];
    const double per = q[1] + q[2] * P + fill * (q[3] + q[4] * P) + shared * q[5];
    return q[0] + nper * (double)rounds * per + q[6] * abits * M * N / 1e6;
}

}  // namespace

// Tile of the matrix-core kernel on packed planes for an M x N output.  Up to 192 tiles of 128 x 128: 64 x 64 tiles on
// two wavefronts, four times as many workgroups (the chip holds 1024 of them at a time, four per compute unit), each
// expanding half the rows: 5 to 15 % faster than 128 x 128 tiles there; at 256 tiles of 128 x 128 the two tie for the
// int8 kind and the larger tile is 10 to 16 % ahead for the fp4 kind on deep products; from 320 on the small tile is 20
// to 50 % slower.  Beyond: 256 x 256 (one workgroup per compute unit) or 128 x 128 (two); a round of 128 x 128 tiles
// over the chip (512 of them) takes 0.67 of a round of 256 x 256 tiles (256 of them) and covers half as much output.
extern "C" int bs_planes_tile(int64_t M, int64_t N, long long *rounds, long long *tiles)
{
    const long long t256 = ((M + 255) / 256) * ((N + 255) / 256), t128 = ((M + 127) / 128) * ((N + 127) / 128);
    if (t128 <= 192) {
        const long long t64 = ((M + 63) / 64) * ((N + 63) / 64);
        if (rounds) *rounds = (t64 + 1023) / 1024;
        if (tiles) *tiles = t64;
        return 64;
    }
    const long long r256 = (t256 + 255) / 256, r128 = (t128 + 511) / 512;
    const bool big = r256 * 100 <= r128 * 67;
    if (rounds) *rounds = big ? r256 : r128;
    if (tiles) *tiles = big ? t256 : t128;
    return big ? 256 : 128;
}

extern "C" bs_engine bs_choose_engine(int wbits, bs_format wfmt, int abits, bs_format afmt, int64_t M, int64_t N, int64_t K)
{
    if (wbits < 1 || wbits > 4 || abits < 1 || abits > 4 || M <= 0 || N <= 0 || K <= 0) return BS_ENGINE_BITSERIAL;
    if ((wfmt == BS_BIPOLAR && wbits != 1) || (afmt == BS_BIPOLAR && abits != 1)) return BS_ENGINE_BITSERIAL;
    if (K >= (int64_t(1) << 30)) return BS_ENGINE_BITSERIAL;  // beyond the dense engines' depth range
    if (N <= 4) return BS_ENGINE_BITSERIAL;  // weights streamed once: wbits/8 byte per weight, nothing to expand
    const double pairs = (double)wbits * abits, kk = (double)K / 1024.0;
    // 5..16 columns: the bit-serial call takes the faster of the streaming kernel in groups of four columns and
    // the tiled kernel with 32 x 8 tiles (the same two models decide inside bs_gemm)
    double t_bitserial = t_bitserial_tiled((double)M, (double)N, (double)K, wbits, abits);
    if (N <= 16) {
        const double groups = (double)((N + 3) / 4) * (double)M / 4096.0;
        const double t_stream = 3.88 + groups * (0.69 + 0.2 * pairs + 0.031 * pairs * kk);
        const double blocks = (double)((M + 31) / 32) * (double)((N + 7) / 8);
        const double rounds = 1.0 + (blocks > 256.0 ? (blocks - 256.0) / 900.0 : 0.0);
        const double t_tiled = 3.64 + rounds * pairs * (0.253 * kk + 0.21);
        t_bitserial = t_stream < t_tiled ? t_stream : t_tiled;
    }
    const bool fp4 = fp4_usable(wbits, abits, K);
    const double t_dense = t_planes((double)M, (double)N, (double)K, wbits, abits, fp4);
    if (t_dense < t_bitserial) return fp4 ? BS_ENGINE_DENSE_FP4 : BS_ENGINE_DENSE_I8;
    return BS_ENGINE_BITSERIAL;
}
