// Pieces shared by the matrix-core kernels (operands already unpacked: bs_dense.hip; operands expanded from
// packed planes inside the loader: bs_planes_mfma.hip): the two operand kinds and their MFMA instruction, the
// parameter block of the epilogue, and the epilogue itself (int32 store, or successive thresholding of
// Sec. 2.1.1 with the packed-plane output).
#pragma once
#include <algorithm>
#include <type_traits>
#include <vector>

#include "bs_common.h"

namespace bs {
namespace dense {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Operand kinds.  I8: one int8 per depth index, v_mfma_i32_32x32x32_i8 (32 depth indices per
// instruction).  FP4: two 4-bit E2M1 floating-point codes per byte (low nibble = even depth index),
// v_mfma_f32_32x32x64_f8f6f4 with both formats set to fp4 (64 depth indices per instruction, the same
// 16 operand bytes per lane, twice the int8 rate); every value of a <= 2-bit operand (and of a 3-bit
// two's-complement one) is an E2M1 number, products and sums stay integers below 2^24, so the fp32
// accumulators are exact and convert to int32 without rounding.  Lane l supplies the 16 bytes
// [16 (l / 32), 16 (l / 32) + 16) of row l % 32 of the instruction's depth step in both kinds, and
// the accumulator layout is the same.
template <bool FP4> struct AccOf { using type = v16i; };
template <> struct AccOf<true> { using type = v16f; };

template <bool FP4>
__device__ __forceinline__ typename AccOf<FP4>::type mma(v4i a, v4i b, typename AccOf<FP4>::type c)
{
    if constexpr (FP4) {
        const v8i a8 = {a.x, a.y, a.z, a.w, 0, 0, 0, 0}, b8 = {b.x, b.y, b.z, b.w, 0, 0, 0, 0};
        // format selectors 4 = fp4 for both operands; zero scale operands select the unscaled instruction
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
}

constexpr int DK = 64;        // depth bytes per row and stage
constexpr int DROW = 80;      // LDS row stride in bytes (64 + 16 pad)
constexpr int DCH = DK / 16;  // 16-byte chunks per row and stage

struct DenseParams {
    const int8_t *W;   // [M][ldw]
    const int8_t *A;   // [N][lda]  (activations, depth-contiguous)
    long long ldw, lda;
    int M, N, K;       // K: depth in operand BYTES (int8: depth indices; fp4: half as many)
    int32_t *C;
    long long ldc;
    const int32_t *thr;
    int T, obits;
    uint32_t *Y;
    int Yd;
    int gx, gy;        // tiles along N and M
    // tile order (plan_tile_order): 0 = workgroup i takes tile i of the row-major order; 1, 2 = the workgroups of an
    // XCD (workgroup index mod 8) take a run of consecutive tiles, xcd_base (+ 1 for the first xcd_rem XCDs) of them,
    // in row-major (1) or column-major (2) order of the tile grid
    int order, xcd_base, xcd_rem;
};

// Tile of the calling workgroup under the order chosen on the host.
__device__ __forceinline__ void tile_of_workgroup(const DenseParams &p, int &tile_m, int &tile_n)
{
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int lin = p.order == 0 ? (int)blockIdx.x : xcd * p.xcd_base + (xcd < p.xcd_rem ? xcd : p.xcd_rem) + local;
    if (p.order == 2) { tile_n = lin / p.gy; tile_m = lin - tile_n * p.gy; }
    else { tile_m = lin / p.gx; tile_n = lin - tile_m * p.gx; }
}

// Which tiles the workgroups of one XCD take.  Workgroups are dealt round-robin to the 8 XCDs, each with its own 4 MiB
// L2, so workgroup i of the plain order lands on XCD i mod 8: with a tile grid whose width is a multiple of 8 an XCD
// then owns a few tile columns and walks down all tile rows (good: its activation panels stay in L2), but with an odd
// width, or few tile rows or columns, every XCD touches nearly every panel of the larger operand (384 x 10816 in 64 x 64
// tiles: 127 of the 169 column panels per XCD, where a run of consecutive tiles in column-major order needs 22).  The
// three orders are compared by walking XCD 0's tiles in launch order, `resident` at a time (what the XCD's compute
// units hold): every panel (a tile's rows of one operand over the whole depth) that was not touched by the previous
// group costs its bytes; if a group's panels exceed the L2, nothing is kept.  Ties keep the plain order.
// w_panel, a_panel: bytes of a tile's weight rows and of its activation rows.
inline void plan_tile_order(DenseParams &p, long long w_panel, long long a_panel, int resident)
{
    const long long blocks = (long long)p.gx * p.gy;
    p.order = 0; p.xcd_base = (int)(blocks / 8); p.xcd_rem = (int)(blocks % 8);
    if (blocks < 16 || blocks > 8192) return;  // small grids have nothing to order; the walk below stays a few microseconds of host time
    const int gx = p.gx, gy = p.gy, n0 = (int)((blocks + 7) / 8);
    long long best = -1;
    std::vector<int> seen_row(gy), seen_col(gx);
    for (int order = 0; order < 3; ++order) {
        std::fill(seen_row.begin(), seen_row.end(), -2);
        std::fill(seen_col.begin(), seen_col.end(), -2);
        long long cost = 0;
        for (int g0 = 0, g = 0; g0 < n0; g0 += resident, ++g) {
            const int g1 = std::min(n0, g0 + resident);
            long long fresh = 0, all = 0;
            for (int local = g0; local < g1; ++local) {
                const long long lin = order == 0 ? 8LL * local : local;
                if (lin >= blocks) break;
                const int tm = order == 2 ? (int)(lin % gy) : (int)(lin / gx), tn = order == 2 ? (int)(lin / gy) : (int)(lin % gx);
                if (seen_row[tm] != g) { all += w_panel; if (seen_row[tm] != g - 1) fresh += w_panel; seen_row[tm] = g; }
                if (seen_col[tn] != g) { all += a_panel; if (seen_col[tn] != g - 1) fresh += a_panel; seen_col[tn] = g; }
            }
            cost += all <= (3LL << 20) ? fresh : all;
        }
        if (best < 0 || cost < best) { best = cost; p.order = order; }
    }
}

// zero the bytes of a 16-byte chunk that lie at or beyond depth index K
__device__ __forceinline__ uint4 mask_tail(uint4 v, int k, int K)
{
    if (k + 16 <= K) return v;
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const int left = K - (k + 4 * d);  // valid bytes in this dword
        if (left <= 0) w[d] = 0;
        else if (left < 4) w[d] &= (1u << (8 * left)) - 1u;
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// Thresholding epilogue for OB output bits (T = 2^OB - 1 thresholds per row, Sec. 2.1.1): the
// tile's thresholds go to LDS (the operand tiles are no longer needed), one row padded to a
// power of two with INT_MAX (never reached, which also zeroes rows past M); every output is
// compared with its row's T thresholds, the count's OB bits are placed at the row's position
// of one 32-row word per plane, and the words leave as whole dwords.
// Turns an accumulator into the int32 product.  The kernels on unpacked operands accumulate the product itself
// (PlainResult); the kernel on packed planes accumulates a product of unsigned codes and adds per-row and per-column
// terms (see bs_planes_mfma.hip).  row, col: position inside the workgroup's tile.
struct PlainResult {
    template <class ACC> __device__ __forceinline__ int operator()(ACC a, int, int) const { return (int)a; }
};

template <int OB, int WTM, int WTN, bool FP4, int WGM, int WGN, class RESULT>
__device__ __forceinline__ void dense_threshold_planes(const DenseParams &p, typename AccOf<FP4>::type (&acc)[WTM][WTN],
                                                       unsigned char *lds, int m0, int n0, const RESULT &result)
{
    constexpr int T = (1 << OB) - 1;
    constexpr int TS = OB == 1 ? 1 : OB == 2 ? 4 : OB == 3 ? 8 : 16;  // table entries per row
    constexpr int BM = 32 * WTM * WGM, NT = 64 * WGM * WGN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int li = lane & 31, lg = lane >> 5;
    __syncthreads();
    int32_t *tl = reinterpret_cast<int32_t *>(lds);  // [BM][TS]
    for (int it = tid; it < BM * TS; it += NT) {
        const int r = it / TS, t = it % TS;
        tl[it] = (m0 + r < p.M && t < T) ? p.thr[(long long)(m0 + r) * T + t] : 0x7fffffff;
    }
    __syncthreads();
#pragma unroll
    for (int a = 0; a < WTM; ++a) {
        const int rbase = (wm * WTM + a) * 32;  // first row of this 32-row band within the block tile
        // Bit-sliced over the lane's 16 rows of the band: hit[b][t] collects one bit per row (compare into the carry,
        // hit = 2 hit + carry, rows taken from the last down so that accumulator v ends up in bit v), a carry-save
        // adder tree turns the T words into the OB plane words of the 16 rows at once, and the 16 bits are spread to
        // the rows' places in the 32-row word: v -> 8 (v / 4) + 4 lg + v % 4.
        uint32_t hit[WTN][T];
#pragma unroll
        for (int b = 0; b < WTN; ++b)
#pragma unroll
            for (int t = 0; t < T; ++t) hit[b][t] = 0;
#pragma unroll
        for (int v = 15; v >= 0; --v) {
            const int rr = 8 * (v >> 2) + 4 * lg + (v & 3);
            // one row's thresholds serve the WTN column tiles this lane holds
            int th[TS];
            if constexpr (TS == 1) {
                th[0] = tl[rbase + rr];
            } else {
#pragma unroll
                for (int q = 0; q < TS / 4; ++q) {
                    const int4 t4 = reinterpret_cast<const int4 *>(tl)[(rbase + rr) * (TS / 4) + q];
                    th[4 * q] = t4.x; th[4 * q + 1] = t4.y; th[4 * q + 2] = t4.z; th[4 * q + 3] = t4.w;
                }
            }
#pragma unroll
            for (int b = 0; b < WTN; ++b) {
                const int c = result(acc[a][b][v], rbase + rr, (wn * WTN + b) * 32 + li);
#pragma unroll
                for (int e = 0; e < T; ++e)
                    asm("v_cmp_le_i32 vcc, %2, %1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(hit[b][e]) : "v"(c), "v"(th[e]) : "vcc");
            }
        }
        uint32_t word[WTN][OB];
#pragma unroll
        for (int b = 0; b < WTN; ++b) {
            count_planes<OB>(hit[b], word[b]);
#pragma unroll
            for (int pl = 0; pl < OB; ++pl) {
                uint32_t x = word[b][pl];                    // 16 bits: nibble g holds rows 8 g + 4 lg .. + 3
                x = (x | (x << 8)) & 0x00FF00FFu;
                x = (x | (x << 4)) & 0x0F0F0F0Fu;
                word[b][pl] = x << (4 * lg);
            }
        }
        // Tiles of a multiple of 128 rows cover at least the Yd words of a column (Yd is a multiple of four), so
        // every word, padding included, is written by some band; words beyond Yd (a 256-row tile over a shorter
        // column) are dropped.  A tile of 64 rows may end two words short of Yd: the last band of the last row
        // tile clears them.
        const int wi = (m0 + rbase) / 32;
        const bool clears_rest = (BM % 128 != 0) && m0 + BM >= p.M && wm == WGM - 1 && a == WTM - 1;
#pragma unroll
        for (int b = 0; b < WTN; ++b) {
            const int n = n0 + (wn * WTN + b) * 32 + li;
            // the two half-wavefronts hold complementary rows of the same column
#pragma unroll
            for (int pl = 0; pl < OB; ++pl) word[b][pl] |= __shfl_xor(word[b][pl], 32);
            if (lg == 0 && n < p.N && wi < p.Yd) {
#pragma unroll
                for (int pl = 0; pl < OB; ++pl) p.Y[((long long)pl * p.N + n) * p.Yd + wi] = word[b][pl];
                if (clears_rest) {
                    for (int z = wi + 1; z < p.Yd; ++z)
#pragma unroll
                        for (int pl = 0; pl < OB; ++pl) p.Y[((long long)pl * p.N + n) * p.Yd + z] = 0;
                }
            }
        }
    }
}

// Epilogue shared by the two dense kernels: int32 store, or successive thresholding with
// the packed-plane output.  `lds` is the (no longer needed) operand space of the caller.
template <int WTM, int WTN, bool FUSE, bool FP4, int WGM = 2, int WGN = 2, class RESULT = PlainResult>
__device__ __forceinline__ void dense_epilogue(const DenseParams &p, typename AccOf<FP4>::type (&acc)[WTM][WTN],
                                               unsigned char *lds, int m0, int n0, int tile_m, const RESULT &result = RESULT())
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int li = lane & 31, lg = lane >> 5;
    (void)tile_m;
    if constexpr (!FUSE) {
        constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN;
        // a tile that lies wholly inside C stores without a test (and without a branch) per element
        const bool inside = m0 + BM <= p.M && n0 + BN <= p.N;  // uniform
#pragma unroll
        for (int a = 0; a < WTM; ++a)
#pragma unroll
            for (int b = 0; b < WTN; ++b) {
                const int n = n0 + (wn * WTN + b) * 32 + li;
                const int mr = (wm * WTM + a) * 32 + 4 * lg;   // this lane's first row of the 32-row band, within the tile
                int32_t *cp = p.C + (long long)(m0 + mr) * p.ldc + n;
                if (inside) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int dr = 8 * (v >> 2) + (v & 3);
                        cp[(long long)dr * p.ldc] = result(acc[a][b][v], mr + dr, n - n0);
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int dr = 8 * (v >> 2) + (v & 3);
                        if (m0 + mr + dr < p.M && n < p.N) cp[(long long)dr * p.ldc] = result(acc[a][b][v], mr + dr, n - n0);
                    }
                }
            }
    } else {
        switch (p.obits) {  // uniform
        case 1: dense_threshold_planes<1, WTM, WTN, FP4, WGM, WGN>(p, acc, lds, m0, n0, result); break;
        case 2: dense_threshold_planes<2, WTM, WTN, FP4, WGM, WGN>(p, acc, lds, m0, n0, result); break;
        case 3: dense_threshold_planes<3, WTM, WTN, FP4, WGM, WGN>(p, acc, lds, m0, n0, result); break;
        default: dense_threshold_planes<4, WTM, WTN, FP4, WGM, WGN>(p, acc, lds, m0, n0, result); break;
        }
    }
}

}  // namespace dense
}  // namespace bs
