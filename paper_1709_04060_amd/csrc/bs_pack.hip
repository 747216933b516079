// Bit-plane packing (Sec. 3.1 of the paper: plane i is the binary matrix of bit i of
// every element; Alg. 1: depth packed into machine words).
//
// The work is a bit-matrix transposition: 64 elements of b bits become b words of 64
// bits.  Both fast kernels do it with SWAR arithmetic on dwords that hold four element
// codes, one per byte:
//   * "vertical" accumulation  acc = (acc << 1) | ((x >> p) & 0x01010101)  over eight
//     such dwords leaves, in each byte of acc, eight consecutive bits of plane p
//     (0.75 VALU ops per element and plane);
//   * a 4 x 4 byte transposition (eight v_perm_b32) brings the bytes into place.
// pack_rows (depth-contiguous source, weights): a thread owns one 64-element word of a
// row, reads it as 4 x 16 bytes, byte-transposes FIRST so that byte lane b of dword i
// holds element 8 b + i, then accumulates vertically: the result is the packed word.
// pack_cols (depth-strided source, activations stored K x N): a thread owns four
// adjacent columns (one dword per depth index, so a wavefront reads full 128-byte
// lines), accumulates vertically along the depth, byte-transposes AFTERWARDS to split
// the four columns, and the workgroup passes the words through LDS so that every
// packed row leaves as a 128-byte (mid-sized inputs: 64-byte) run.
// Generic one-element-per-lane kernels cover unaligned sources.
#include "bs_common.h"

namespace {

constexpr uint32_t kLsbOfBytes = 0x01010101u;

// t_b = [a0.byte b, a1.byte b, a2.byte b, a3.byte b]  (byte 0 first)
__device__ __forceinline__ void transpose_bytes_4x4(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3,
                                                    uint32_t &t0, uint32_t &t1, uint32_t &t2, uint32_t &t3)
{
    // __builtin_amdgcn_perm(hi, lo, sel): selector values 0..3 take bytes of lo, 4..7 of hi
    const uint32_t p01_lo = __builtin_amdgcn_perm(a1, a0, 0x05010400u);  // a0.0 a1.0 a0.1 a1.1
    const uint32_t p01_hi = __builtin_amdgcn_perm(a1, a0, 0x07030602u);  // a0.2 a1.2 a0.3 a1.3
    const uint32_t p23_lo = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
    const uint32_t p23_hi = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
    t0 = __builtin_amdgcn_perm(p23_lo, p01_lo, 0x05040100u);
    t1 = __builtin_amdgcn_perm(p23_lo, p01_lo, 0x07060302u);
    t2 = __builtin_amdgcn_perm(p23_hi, p01_hi, 0x05040100u);
    t3 = __builtin_amdgcn_perm(p23_hi, p01_hi, 0x07060302u);
}

// Four int8 values in a dword -> four codes, one per byte.  Unsigned and two's
// complement codes are the low bits of the value itself (only bits < `bits` are ever
// read).  Bipolar: code = (v > 0), per byte: nonzero and sign bit clear.
template <bool BIP>
__device__ __forceinline__ uint32_t codes_of_i8x4(uint32_t x)
{
    if (!BIP) return x;
    const uint32_t nonzero = ((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x;  // bit 7 of a byte set iff the byte != 0
    return ((nonzero & ~x) >> 7) & kLsbOfBytes;
}

template <bool BIP>
__device__ __forceinline__ uint32_t codes_of_i32x4(int v0, int v1, int v2, int v3)
{
    if (BIP) return (uint32_t)(v0 > 0) | ((uint32_t)(v1 > 0) << 8) | ((uint32_t)(v2 > 0) << 16) | ((uint32_t)(v3 > 0) << 24);
    return ((uint32_t)v0 & 0xFFu) | (((uint32_t)v1 & 0xFFu) << 8) | (((uint32_t)v2 & 0xFFu) << 16) | ((uint32_t)v3 << 24);
}

// Eight dwords of codes -> for plane p a dword whose byte b, bit i is bit p of byte b of x[i].
__device__ __forceinline__ uint32_t vertical8(const uint32_t (&x)[8], int p)
{
    uint32_t acc = 0;
#pragma unroll
    for (int i = 7; i >= 0; --i) acc = (acc << 1) | ((x[i] >> p) & kLsbOfBytes);
    return acc;
}

// ------------------------------------------------------------------ pack_rows (fast)
// One thread per (row, word).  T = int8_t: the word's 64 bytes are 4 x uint4.
template <typename T, bool BIP>
__global__ void __launch_bounds__(256)
pack_rows_kernel(const T *__restrict__ src, int64_t rows, int64_t depth, int64_t ld, int bits,
                 uint64_t *__restrict__ planes, int64_t S)
{
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= rows * S) return;
    const int64_t r = item / S, d = item - r * S;
    const int64_t k0 = d * 64;
    const T *row = src + r * ld;

    uint32_t L[16];  // L[j] = codes of elements k0 + 4 j .. k0 + 4 j + 3
    if (k0 + 64 <= depth) {
        if constexpr (sizeof(T) == 1) {
            const uint4 *q = reinterpret_cast<const uint4 *>(row + k0);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint4 v = q[c];
                L[4 * c + 0] = codes_of_i8x4<BIP>(v.x); L[4 * c + 1] = codes_of_i8x4<BIP>(v.y);
                L[4 * c + 2] = codes_of_i8x4<BIP>(v.z); L[4 * c + 3] = codes_of_i8x4<BIP>(v.w);
            }
        } else {
            const int4 *q = reinterpret_cast<const int4 *>(row + k0);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int4 v = q[j];
                L[j] = codes_of_i32x4<BIP>(v.x, v.y, v.z, v.w);
            }
        }
    } else {  // the last, partial word of a row (or a pure padding word): element by element
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            int v[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int64_t k = k0 + 4 * j + b;
                v[b] = k < depth ? (int)row[k] : 0;
            }
            L[j] = codes_of_i32x4<BIP>(v[0], v[1], v[2], v[3]);
        }
    }

    uint32_t w[2][bs::kMaxBits];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        // X[i].byte b = element 32 h + 8 b + i
        uint32_t X[8];
        transpose_bytes_4x4(L[8 * h + 0], L[8 * h + 2], L[8 * h + 4], L[8 * h + 6], X[0], X[1], X[2], X[3]);
        transpose_bytes_4x4(L[8 * h + 1], L[8 * h + 3], L[8 * h + 5], L[8 * h + 7], X[4], X[5], X[6], X[7]);
#pragma unroll
        for (int p = 0; p < bs::kMaxBits; ++p) w[h][p] = (p < bits) ? vertical8(X, p) : 0u;
    }
#pragma unroll
    for (int p = 0; p < bs::kMaxBits; ++p)
        if (p < bits) planes[((int64_t)p * rows + r) * S + d] = ((uint64_t)w[1][p] << 32) | w[0][p];
}

// ------------------------------------------------------------------ pack_cols (fast)
// Workgroup tile: 128 rows (= source columns n) x 8 words (512 depth indices).
// Thread (tx, ty): rows 4 tx .. 4 tx + 3, word ty.  The planes of the tile pass through LDS
// (bits x 8 KiB, sized at launch) so that they leave as 64-byte runs per (plane, row).
// A tile of twice the depth (128-byte runs) measured slower at every size: the smaller
// tile keeps more workgroups resident per compute unit.
constexpr int PC_ROWS = 128;
constexpr int PC_WORDS = 8;
constexpr int PC_PAIRS = PC_WORDS / 2;  // 16-byte slots per row of the LDS tile

template <typename T, bool BIP>
__global__ void __launch_bounds__(256)
pack_cols_kernel(const T *__restrict__ src, int64_t rows, int64_t depth, int64_t ld, int bits,
                 uint64_t *__restrict__ planes, int64_t S)
{
    // [plane][row][PC_PAIRS pairs of words], pair slot XOR-swizzled with (row / 4) & (PC_PAIRS - 1)
    extern __shared__ uint4 tile[];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int64_t r0 = (int64_t)blockIdx.x * PC_ROWS;
    const int64_t d0 = (int64_t)blockIdx.y * PC_WORDS;
    const int64_t rq = r0 + 4 * tx;                 // first of this thread's four rows
    const bool full_quad = rq + 4 <= rows;

    uint32_t out[bs::kMaxBits][4][2];               // [plane][row of the quad][lo/hi dword]
    const int64_t kw = (d0 + ty) * 64;              // first depth index of the word
    uint32_t A[bs::kMaxBits][8];                    // [plane][group of 8 depth indices]
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        uint32_t X[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int64_t k = kw + 8 * g + i;
            uint32_t x = 0;
            if (k < depth) {
                const T *e = src + k * ld + rq;
                if (full_quad) {
                    if constexpr (sizeof(T) == 1) x = codes_of_i8x4<BIP>(*reinterpret_cast<const uint32_t *>(e));
                    else {
                        const int4 v = *reinterpret_cast<const int4 *>(e);
                        x = codes_of_i32x4<BIP>(v.x, v.y, v.z, v.w);
                    }
                } else {
                    int v[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) v[b] = (rq + b < rows) ? (int)e[b] : 0;
                    x = codes_of_i32x4<BIP>(v[0], v[1], v[2], v[3]);
                }
            }
            X[i] = x;
        }
#pragma unroll
        for (int p = 0; p < bs::kMaxBits; ++p) A[p][g] = (p < bits) ? vertical8(X, p) : 0u;
    }
    // A[p][g].byte c = bits 8 g .. 8 g + 7 of row c: split the four rows
#pragma unroll
    for (int p = 0; p < bs::kMaxBits; ++p) {
        transpose_bytes_4x4(A[p][0], A[p][1], A[p][2], A[p][3], out[p][0][0], out[p][1][0], out[p][2][0], out[p][3][0]);
        transpose_bytes_4x4(A[p][4], A[p][5], A[p][6], A[p][7], out[p][0][1], out[p][1][1], out[p][2][1], out[p][3][1]);
    }
#pragma unroll
    for (int p = 0; p < bs::kMaxBits; ++p)
        if (p < bits) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {  // one word: half of the pair slot (ty >> 1)
                uint2 *slot = reinterpret_cast<uint2 *>(
                    &tile[(p * PC_ROWS + 4 * tx + c) * PC_PAIRS + ((ty >> 1) ^ (tx & (PC_PAIRS - 1)))]);
                slot[ty & 1] = make_uint2(out[p][c][0], out[p][c][1]);
            }
        }
    __syncthreads();
    // write out: PC_PAIRS consecutive threads cover the contiguous run of one (plane, row)
    const int pair = threadIdx.x & (PC_PAIRS - 1);
    for (int p = 0; p < bits; ++p)
        for (int rr = threadIdx.x / PC_PAIRS; rr < PC_ROWS; rr += 256 / PC_PAIRS) {
            const int64_t r = r0 + rr, d = d0 + 2 * pair;
            if (r < rows && d < S)
                *reinterpret_cast<uint4 *>(planes + ((int64_t)p * rows + r) * S + d) =
                    tile[(p * PC_ROWS + rr) * PC_PAIRS + (pair ^ ((rr >> 2) & (PC_PAIRS - 1)))];
        }
}

// ------------------------------------------------------------------ generic kernels
template <typename T>
__device__ __forceinline__ uint32_t encode(T v, int bits, int bipolar)
{
    const int x = static_cast<int>(v);
    return bipolar ? static_cast<uint32_t>(x > 0) : (static_cast<uint32_t>(x) & ((1u << bits) - 1u));
}

// One wavefront per (row, word): a 64-lane ballot of bit p IS the packed word of plane p.
template <typename T>
__global__ void __launch_bounds__(256)
pack_rows_generic(const T *__restrict__ src, int64_t rows, int64_t depth, int64_t ld, int bits, int bipolar,
                  uint64_t *__restrict__ planes, int64_t S)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    const int64_t items = rows * S;
    for (int64_t it = wave; it < items; it += nwaves) {
        const int64_t r = it / S, d = it - r * S;
        const int64_t k = d * 64 + lane;
        uint32_t code = 0;
        if (k < depth) code = encode(src[r * ld + k], bits, bipolar);
        uint64_t mine = 0;
        for (int p = 0; p < bits; ++p) {
            const uint64_t word = __ballot((code >> p) & 1u);
            if (lane == p) mine = word;
        }
        if (lane < bits) planes[((int64_t)lane * rows + r) * S + d] = mine;
    }
}

// Block = 64 rows (lanes) x 4 words (wavefronts).  Element (r, k) at src[k * ld + r].
template <typename T>
__global__ void __launch_bounds__(256)
pack_cols_generic(const T *__restrict__ src, int64_t rows, int64_t depth, int64_t ld, int bits, int bipolar,
                  uint64_t *__restrict__ planes, int64_t S)
{
    const int64_t r = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
    const int64_t d = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
    if (r >= rows || d >= S) return;
    uint64_t w[bs::kMaxBits] = {0, 0, 0, 0};
    const int64_t k0 = d * 64;
    const int kn = (int)(depth - k0 < 64 ? (depth - k0 < 0 ? 0 : depth - k0) : 64);
    for (int kk = 0; kk < kn; ++kk) {
        const uint32_t code = encode(src[(k0 + kk) * ld + r], bits, bipolar);
#pragma unroll
        for (int p = 0; p < bs::kMaxBits; ++p) w[p] |= (uint64_t)((code >> p) & 1u) << kk;
    }
    for (int p = 0; p < bits; ++p) planes[((int64_t)p * rows + r) * S + d] = w[p];
}

template <typename T>
bs_status launch_pack(const T *src, int64_t rows, int64_t depth, int64_t ld, int strided, int bits, bool bip,
                      uint64_t *planes, int64_t S, hipStream_t st)
{
    // the fast kernels read 16 bytes (rows) resp. four elements (cols) at a time
    const size_t row_align = 16, quad_align = 4 * sizeof(T);
    if (!strided) {
        const bool fast = bs::aligned(src, row_align) && (ld * sizeof(T)) % row_align == 0;
        if (fast) {
            const int64_t blocks = (rows * S + 255) / 256;
            if (blocks >= (int64_t(1) << 31)) return BS_ERR_OVERFLOW_RISK;
            if (bip) pack_rows_kernel<T, true><<<dim3((unsigned)blocks), 256, 0, st>>>(src, rows, depth, ld, bits, planes, S);
            else pack_rows_kernel<T, false><<<dim3((unsigned)blocks), 256, 0, st>>>(src, rows, depth, ld, bits, planes, S);
        } else {
            int64_t blocks = (rows * S + 3) / 4;
            if (blocks > 256 * 64) blocks = 256 * 64;
            pack_rows_generic<T><<<dim3((unsigned)blocks), 256, 0, st>>>(src, rows, depth, ld, bits, bip, planes, S);
        }
    } else {
        const bool fast = bs::aligned(src, quad_align) && (ld * sizeof(T)) % quad_align == 0;
        if (fast) {
            dim3 grid((unsigned)((rows + PC_ROWS - 1) / PC_ROWS), (unsigned)((S + PC_WORDS - 1) / PC_WORDS));
            if (grid.y > 65535) return BS_ERR_OVERFLOW_RISK;
            const size_t lds = (size_t)bits * PC_ROWS * PC_PAIRS * sizeof(uint4);
            if (bip) pack_cols_kernel<T, true><<<grid, 256, lds, st>>>(src, rows, depth, ld, bits, planes, S);
            else pack_cols_kernel<T, false><<<grid, 256, lds, st>>>(src, rows, depth, ld, bits, planes, S);
        } else {
            dim3 grid((unsigned)((rows + 63) / 64), (unsigned)((S + 3) / 4));
            if (grid.y > 65535) return BS_ERR_OVERFLOW_RISK;
            pack_cols_generic<T><<<grid, 256, 0, st>>>(src, rows, depth, ld, bits, bip, planes, S);
        }
    }
    return bs::after_launch();
}

}  // namespace

extern "C" int64_t bs_words_per_row(int64_t depth) { return depth <= 0 ? 0 : 2 * ((depth + 127) / 128); }

extern "C" bs_status bs_pack_planes(const void *src, bs_dtype dtype, int64_t rows, int64_t depth, int64_t ld,
                                    int depth_is_strided, int bits, bs_format fmt, uint64_t *planes, void *stream)
{
    if (!src || !planes || rows <= 0 || depth <= 0) return BS_ERR_INVALID_ARG;
    if (dtype != BS_I8 && dtype != BS_I32) return BS_ERR_INVALID_ARG;
    if (bs_status s = bs::check_bits_fmt(bits, fmt)) return s;
    if (ld < (depth_is_strided ? rows : depth)) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(planes, 16)) return BS_ERR_ALIGNMENT;
    if (dtype == BS_I32 && !bs::aligned(src, 4)) return BS_ERR_ALIGNMENT;
    const int64_t S = bs_words_per_row(depth);
    if (rows * S * 2 >= (int64_t(1) << 31)) return BS_ERR_OVERFLOW_RISK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bip = fmt == BS_BIPOLAR;
    if (dtype == BS_I8)
        return launch_pack(static_cast<const int8_t *>(src), rows, depth, ld, depth_is_strided, bits, bip, planes, S, st);
    return launch_pack(static_cast<const int32_t *>(src), rows, depth, ld, depth_is_strided, bits, bip, planes, S, st);
}
