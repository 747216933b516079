// Rate probe for the instruction pair the bit-serial inner loop is made of (Alg. 1: AND, then
// popcount-accumulate).  Register operands only, no memory traffic: what it measures is the
// ceiling the chip sustains for v_and_b32 + v_bcnt_u32_b32 at the clock it holds under this load,
// the measured counterpart of the theoretical VALU popcount peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bs_common.h"
#include "bsgemm.h"

namespace {

// Eight products per statement: AND, popcount-accumulate, one idle issue slot.  A SIMD executes the AND
// in two cycles and the popcount in four while one wavefront issues at most every four cycles; the idle
// slot is what lets several resident wavefronts interleave (measured: 48.8e12 lane-operations per second
// with the slot and eight wavefronts per SIMD, 39.5e12 without it).
// Operands: %0 %1 temporaries, %2..%9 accumulators, %10 %11 weight words, %12..%15 activation words.
#define BS_PROBE_STEP(T, ACC, W, A) "v_and_b32 %" #T ", %" #W ", %" #A "\n\tv_bcnt_u32_b32 %" #ACC ", %" #T ", %" #ACC "\n\ts_nop 0\n\t"

__device__ __forceinline__ void eight_products(uint32_t *acc, uint32_t w0, uint32_t w1, const uint32_t *a)
{
    uint32_t t0, t1;
    asm volatile(BS_PROBE_STEP(0, 2, 10, 12) BS_PROBE_STEP(1, 3, 10, 13) BS_PROBE_STEP(0, 4, 10, 14) BS_PROBE_STEP(1, 5, 10, 15)
                 BS_PROBE_STEP(0, 6, 11, 12) BS_PROBE_STEP(1, 7, 11, 13) BS_PROBE_STEP(0, 8, 11, 14) BS_PROBE_STEP(1, 9, 11, 15)
                 : "=&v"(t0), "=&v"(t1), "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]),
                   "+v"(acc[6]), "+v"(acc[7])
                 : "v"(w0), "v"(w1), "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]));
}

// 4 x 4 accumulators per lane, as in the GEMM's lane tile: per pass 16 ANDs and 16 popcount-adds.
__global__ void __launch_bounds__(256) popcount_rate_kernel(uint32_t *sink, int passes)
{
    uint32_t w[4], a[4], acc[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        w[i] = 0x9e3779b9u * (threadIdx.x + 17 * i + 1);
        a[i] = 0x85ebca6bu * (blockIdx.x + 29 * i + 1) ^ threadIdx.x;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0;
    for (int it = 0; it < passes; it += 4) {  // four passes per trip keep the loop's own instructions below 2 %
        eight_products(acc, w[0], w[1], a);
        eight_products(acc + 8, w[2], w[3], a);
        eight_products(acc, w[1], w[2], a);
        eight_products(acc + 8, w[3], w[0], a);
        eight_products(acc, w[2], w[3], a);
        eight_products(acc + 8, w[0], w[1], a);
        eight_products(acc, w[3], w[0], a);
        eight_products(acc + 8, w[1], w[2], a);
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s ^= acc[i];
    if (threadIdx.x == 0) sink[blockIdx.x] = s;
}

// Streaming read: every lane XORs 16-byte loads of a contiguous buffer, four in flight per lane, a workgroup per
// 16 KiB slice round-robin over the grid; the workgroup stores one word so that the loads are observable.  NT: with
// the non-temporal hint.
template <bool NT>
__global__ void __launch_bounds__(256) stream_read_kernel(const uint4 *__restrict__ src, long long chunks, uint32_t *sink)
{
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    uint32_t s = 0;
    for (long long base = (long long)blockIdx.x * 1024; base < chunks; base += (long long)gridDim.x * 1024) {
        v4u v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long long c = base + u * 256 + threadIdx.x;
            v[u] = (v4u){0, 0, 0, 0};
            if (c < chunks) {
                const v4u *q = reinterpret_cast<const v4u *>(src + c);
                v[u] = NT ? __builtin_nontemporal_load(q) : *q;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) s ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s ^= __shfl_xor(s, o);
    if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], s);
}

}  // namespace

extern "C" bs_status bs_probe_stream_read(const void *src, int64_t bytes, uint32_t *sink, int workgroups, int non_temporal,
                                          void *stream)
{
    if (!src || !sink || bytes <= 0 || (bytes & 15) || workgroups <= 0) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(src, 16) || !bs::aligned(sink, 4)) return BS_ERR_ALIGNMENT;
    const long long chunks = bytes / 16;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (non_temporal) stream_read_kernel<true><<<dim3((unsigned)workgroups), 256, 0, st>>>(static_cast<const uint4 *>(src), chunks, sink);
    else stream_read_kernel<false><<<dim3((unsigned)workgroups), 256, 0, st>>>(static_cast<const uint4 *>(src), chunks, sink);
    return bs::after_launch();
}

extern "C" bs_status bs_probe_popcount_rate(uint32_t *sink, int workgroups, int passes, void *stream)
{
    if (!sink || workgroups <= 0 || passes <= 0 || passes % 4 != 0) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(sink, 4)) return BS_ERR_ALIGNMENT;
    popcount_rate_kernel<<<dim3((unsigned)workgroups), 256, 0, static_cast<hipStream_t>(stream)>>>(sink, passes);
    return bs::after_launch();
}
