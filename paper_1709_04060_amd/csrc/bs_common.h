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

// Sum of T = 2^OB - 1 one-bit inputs, bit-sliced: bit i of hit[t] says whether element i reached threshold t; plane
// word w[p] gets bit p of every element's count (Sec. 2.1.1: the activation is the number of thresholds reached).  A
// carry-save adder tree of full adders (two three-input bit operations each): 1, 4 or 11 of them for 32 elements.
__device__ __forceinline__ void full_add(uint32_t x, uint32_t y, uint32_t z, uint32_t &sum, uint32_t &carry)
{
    sum = x ^ y ^ z;
    carry = (x & y) | (z & (x ^ y));
}

template <int OB>
__device__ __forceinline__ void count_planes(const uint32_t (&hit)[(1 << OB) - 1], uint32_t (&w)[OB])
{
    if constexpr (OB == 1) {
        w[0] = hit[0];
    } else if constexpr (OB == 2) {
        full_add(hit[0], hit[1], hit[2], w[0], w[1]);
    } else {
        constexpr int G = ((1 << OB) - 1) / 3;  // full adders of the first level: 2 (7 inputs) or 5 (15 inputs)
        uint32_t s1[G], c1[G];
#pragma unroll
        for (int g = 0; g < G; ++g) full_add(hit[3 * g], hit[3 * g + 1], hit[3 * g + 2], s1[g], c1[g]);
        if constexpr (OB == 3) {
            uint32_t c2;
            full_add(s1[0], s1[1], hit[6], w[0], c2);
            full_add(c1[0], c1[1], c2, w[1], w[2]);
        } else {
            uint32_t t0, c5, c6, u0, u1, d0, d1, d2;
            full_add(s1[0], s1[1], s1[2], t0, c5);
            full_add(t0, s1[3], s1[4], w[0], c6);
            full_add(c1[0], c1[1], c1[2], u0, d0);
            full_add(c1[3], c1[4], c5, u1, d1);
            full_add(u0, u1, c6, w[1], d2);
            full_add(d0, d1, d2, w[2], w[3]);
        }
    }
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
