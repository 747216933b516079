// Internal helpers shared by the HIP translation units of libbsgemm (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bsgemm.h"

namespace bs {

constexpr int kWave = 64;        // CDNA4 wavefront width
constexpr int kMaxBits = 4;      // the few-bit range of the paper (w, a <= 4)

// Output grids at which the bit-serial launch changes its tile (bs_gemm_kernel.h, launch_planes); the time model of the
// engine choice (bs_misc.cpp) follows the same steps.
constexpr long long kNarrowMaxTiles32 = 200;  // measured, W1A2..W4A4 at depth 2048: 32 x 8 tiles win up to 184 tiles of 32 x 32, tie at 256, lose from 512
constexpr long long kHalfWidthMaxTiles32 = 384;  // 32 x 16 tiles between the tiny grids and this many 32 x 32 tiles
constexpr long long kWideMinTiles64 = 512;  // 64 x 64 tiles from this many on, 32 x 32 tiles with the depth split below

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// A kernel's parameter block arrives through scalar loads, and the compiler requests each
// field where it is first needed: for a 350-byte block that is up to nine load-and-wait
// rounds on the serial path of every workgroup.  Touching every 64-byte line of the block in
// one burst at the kernel's entry lets the later field loads hit the scalar cache (measured on
// the small latency-bound layers: 0.1 to 0.3 us per launch).
template <int BYTES>
__device__ __forceinline__ void prefetch_kernel_arguments()
{
    typedef const uint32_t __attribute__((address_space(4))) *karg_ptr;
    karg_ptr ka = (karg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t sink = ka[(BYTES - 4) / 4];
#pragma unroll
    for (int o = 0; o + 4 <= BYTES; o += 64) sink ^= ka[o / 4];
    asm volatile("" ::"s"(sink));  // keeps the loads; nothing is done with the value
}

inline bs_status after_launch() { return hipGetLastError() == hipSuccess ? BS_OK : BS_ERR_LAUNCH; }

inline bs_status check_bits_fmt(int bits, bs_format fmt)
{
    if (bits < 1) return BS_ERR_INVALID_ARG;
    if (fmt != BS_UNSIGNED && fmt != BS_TWOS_COMPLEMENT && fmt != BS_BIPOLAR) return BS_ERR_INVALID_ARG;
    if (fmt == BS_BIPOLAR && bits != 1) return BS_ERR_INVALID_ARG;
    if (bits > kMaxBits) return BS_ERR_UNSUPPORTED;
    return BS_OK;
}

// Largest magnitude a value of this format can take.
inline int64_t max_abs(int bits, bs_format fmt)
{
    if (fmt == BS_BIPOLAR) return 1;
    if (fmt == BS_TWOS_COMPLEMENT) return int64_t(1) << (bits - 1);
    return (int64_t(1) << bits) - 1;
}

}  // namespace bs
