// Status strings and version of libbsgemm.
#include "bsgemm.h"

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

// Per-layer engine choice (Sec. 4.1.1 / 4.2): the faster of the two engines under a time model whose
// constants were fitted to measurements of both engines over M, N in 256..4096, K in {1024, 4096} and
// W1A1, W1A2, W2A2, W4A4 on MI355X (fused 2^abits-level epilogue, activation unpack counted for the
// dense engine; least squares on the logarithm of the time: rms error 11 % and 8 %; over the 144
// measured cases the choice costs 0.3 % on average and 17 % at worst against always picking the faster).
// Microseconds.
extern "C" bs_engine bs_choose_engine(int wbits, int abits, int64_t M, int64_t N, int64_t K)
{
    if (wbits < 1 || wbits > 4 || abits < 1 || abits > 4 || M <= 0 || N <= 0 || K <= 0) return BS_ENGINE_BITSERIAL;
    if (N <= 4) return BS_ENGINE_BITSERIAL;  // weights streamed once: wbits/8 byte per weight beats one byte
    const double pairs = (double)wbits * abits, kk = (double)K / 1024.0;
    const double mnk2 = 2.0 * (double)M * (double)N * (double)K;
    const double t_bitserial = 5.0 + 0.565 * kk * pairs + mnk2 * pairs / 1.27e15 * 1e6;
    const double t_dense = 8.5 + 4.7 * kk + 1.8 * abits + mnk2 / 3.38e15 * 1e6 + (double)M * (double)N / 0.75e12 * 1e6;
    return t_dense < t_bitserial ? BS_ENGINE_DENSE_I8 : BS_ENGINE_BITSERIAL;
}
