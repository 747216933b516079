// Matrix-core engine on PACKED PLANES: the product W . A of Sec. 3.1 computed with MFMA
// instructions from the same bit-plane operands the AND-popcount kernels take.  This is the
// byte-wise engine of the paper's per-layer choice (Sec. 4.1.1, 4.2) without its cost in memory:
// operands stay w/8 and a/8 byte per element in device memory, nothing unpacked is ever written
// there, and no extra buffer or launch is needed.  The loader of the kernel turns plane bits into
// operand codes on their way to LDS:
//   fp4 kind   operands of at most 2 bits; v_mfma_f32_32x32x64_f8f6f4 on 4-bit E2M1 floating-point
//              codes, 128 depth indices per 64-byte LDS row and stage;
//   int8 kind  operands of up to 4 bits; v_mfma_i32_32x32x32_i8, 64 depth indices per row and stage.
//
// What makes the expansion cheap (it runs on the vector unit, and a SIMD does not execute vector and
// matrix instructions at the same time: measured, 16 simple vector instructions behind every matrix
// instruction double the time of a matrix-only loop).
//  1. Unsigned codes, corrected afterwards.  Every format is an affine function of an unsigned code u:
//     unsigned v = u; two's complement v = u - T with u = code xor T, T = 2^(bits-1) (top plane
//     inverted); bipolar v = 2 u - 1.  With v_w = aw u_w + bw and v_a = aa u_a + ba,
//       C[m][n] = aw aa (U_w . U_a)[m][n] + aw ba rowsum(U_w)[m] + bw aa rowsum(U_a)[n] + bw ba K,
//     and the row sums are weighted popcounts of the planes the loader moves anyway (the same trick as
//     the popcount correction of the AND-popcount kernels for bipolar operands).  So the matrix
//     instruction only ever sees unsigned codes, whose bits ARE the plane bits: no table look-up.
//     In the E2M1 format the codes 0000..0011 are 0, 0.5, 1, 1.5, i.e. linear in their two low bits: a
//     2-bit code in the low bits of a nibble is the number u / 2 (a 1-bit operand goes to bit 1 and is
//     u itself); the factor is taken out again when the exact fp32 sum is converted.
//  2. Any order of the depth indices.  The contraction runs over matching positions of the two
//     operands, so the loader may place the indices of a 32-index word in whatever order is cheapest,
//     as long as both operands use the same one.  The planes of a word are merged with masks and
//     shifts (even- and odd-indexed bits first, then pairs of 2-bit fields), which leaves the codes in
//     a fixed permuted order, and they are stored as they come: 12 vector instructions per 32 codes
//     for two planes to nibbles, 36 for four planes to bytes.
// Padding bits are zero in every plane, hence zero codes, except in an inverted top plane, which is
// masked with "index < K".
//
// Pipeline.  A thread owns one row of the stacked [W rows; A rows] tile.  Four LDS stage buffers of 64-byte rows
// (16-byte chunks XOR-swizzled with (row / 4) % 4, the layout of the direct-to-LDS dense kernel, which keeps the fragment
// reads apart in the banks; the threads own the rows in an order that does the same for their row-wise writes): a period of two stages is multiplied
// from two of them while the next period's stages are expanded into the other two, with one barrier per period.
// Plane words are requested a period ahead, 16 bytes per row and plane: every lane of such a request touches
// another cache line, and those look-ups bound the loader (with all lanes on one row the W4A4 8192^3 product took
// 555 instead of 1105 us), hence as few and as wide requests as the registers allow.
#include "bs_dense_common.h"
#include "bs_gemm_kernel.h"

namespace bs {
namespace {

using namespace bs::dense;
typedef __attribute__((address_space(3))) void lds_void;

struct OperandCoding {
    int bits;
    int shift;              // slot of plane 0 (fp4 kind: 2 - bits, so that a 1-bit operand sits in the nibble's bit 1)
    int top;                // slot whose plane is inverted (two's complement), or -1
};

struct PlanesParams {
    DenseParams d;          // epilogue fields (M, N, C, ldc, thr, T, obits, Y, Yd, gx, gy); W, A, ld*, K unused
    const uint32_t *Wp;     // [wbits][M][Kd]
    const uint32_t *Ap;     // [abits][N][Kd]
    int Kd;                 // dwords per packed row
    OperandCoding cw, ca;
    int K32;                // depth in indices (below 2^30)
    int nst;                // stages: ceil(K / indices per stage)
    int nper;               // periods of two stages: ceil(nst / 2)
    // C = mul * P + row_coef * rowsum(U_w)[m] + row_const + col_coef * rowsum(U_a)[n],  P = acc * acc_scale = U_w . U_a
    int mul, row_coef, row_const, col_coef;
    float acc_scale;
    // implicit lowering (CONV kernels): Ap points at packed HWC image planes; see PlanesGemm
    int cH, cW, cCd, cPix, cKW, cStride, cPad, cOW, cOHW, cB, cKused;
};

// (a & m) | (b & ~m): one v_bfi_b32
__device__ __forceinline__ uint32_t bitsel(uint32_t m, uint32_t a, uint32_t b) { return (a & m) | (b & ~m); }

// Even- and odd-indexed bits of two planes merged into 2-bit fields (lo | hi << 1): 16 fields per word each.
// (hi & 0x55..) << 1 is (hi << 1) under the complementary mask, so each merge is a shift and a bit select.
__device__ __forceinline__ void merge_pair(uint32_t lo, uint32_t hi, uint32_t &even, uint32_t &odd)
{
    even = bitsel(0x55555555u, lo, hi << 1);
    odd = bitsel(0x55555555u, lo >> 1, hi);
}

// 32 depth indices of two planes -> 32 nibbles 00 hi lo (16 bytes), in the loader's fixed order of the indices
__device__ __forceinline__ uint4 expand32_fp4(uint32_t lo, uint32_t hi)
{
    uint32_t e, o;
    merge_pair(lo, hi, e, o);
    asm("" : "+v"(e), "+v"(o));  // used as they are: see expand32_i8
    return make_uint4(e & 0x33333333u, (e >> 2) & 0x33333333u, o & 0x33333333u, (o >> 2) & 0x33333333u);
}

// 32 depth indices of four planes -> 32 bytes 0000 x3 x2 x1 x0 (two 16-byte chunks), in the loader's fixed order
__device__ __forceinline__ void expand32_i8(const uint32_t (&x)[4], uint4 &out0, uint4 &out1)
{
    uint32_t e01, o01, e23, o23;
    merge_pair(x[0], x[1], e01, o01);
    merge_pair(x[2], x[3], e23, o23);
    uint32_t n[4];  // 8 nibble codes each: fields of planes 0-1 in the low half of every nibble, of planes 2-3 above
    n[0] = bitsel(0x33333333u, e01, e23 << 2);
    n[1] = bitsel(0x33333333u, e01 >> 2, e23);
    n[2] = bitsel(0x33333333u, o01, o23 << 2);
    n[3] = bitsel(0x33333333u, o01 >> 2, o23);
    // The outputs below take the n[] as they are.  Left transparent, each masked output is rebuilt from the planes'
    // words through a chain of its own that keeps only the bits it needs (52 instead of 36 instructions per 32 codes).
    asm("" : "+v"(n[0]), "+v"(n[1]), "+v"(n[2]), "+v"(n[3]));
    out0 = make_uint4(n[0] & 0x0F0F0F0Fu, (n[0] >> 4) & 0x0F0F0F0Fu, n[1] & 0x0F0F0F0Fu, (n[1] >> 4) & 0x0F0F0F0Fu);
    out1 = make_uint4(n[2] & 0x0F0F0F0Fu, (n[2] >> 4) & 0x0F0F0F0Fu, n[3] & 0x0F0F0F0Fu, (n[3] >> 4) & 0x0F0F0F0Fu);
}

// accumulator -> int32 product: scale out the E2M1 half steps, then the affine terms of the two formats
struct PlanesResult {
    int mul;
    float acc_scale;
    const int *row_term, *col_term;  // LDS, indexed by the row / column inside the tile
    __device__ __forceinline__ int operator()(float a, int row, int col) const
    {
        // one multiplication: mul is 1, 2 or 4 and the scaled sum an integer below 2^24, so the product is exact in fp32
        return wrap_add((int)(a * (acc_scale * (float)mul)), wrap_add(row_term[row], col_term[col]));
    }
    __device__ __forceinline__ int operator()(int a, int row, int col) const
    {
        return wrap_add(wrap_mul(mul, a), wrap_add(row_term[row], col_term[col]));
    }
};

// FP4: operand kind.  WTM x WTN MFMA tiles of 32 x 32 per wavefront, WGM x WGN wavefronts; the workgroup has as many
// threads as the stacked tile has rows (one row per thread).
// CONV: the activation operand is not a packed matrix but packed HWC image planes; the rows of the A part of the tile
// (columns of the lowered matrix of Sec. 3.2) are gathered from the image, zero words for taps outside of it, so
// the lowered matrix never exists in memory.  VEC: a pixel's channel run is a whole number of 16-byte chunks, so that
// four consecutive lowered dwords lie inside one tap of one pixel and are gathered with one load.
template <bool FP4, int WTM, int WTN, int WGM, int WGN, bool FUSE, bool CONV = false, bool VEC = false>
__global__ void __launch_bounds__(64 * WGM * WGN)
planes_mfma_kernel(const PlanesParams p)
{
    constexpr int NB = FP4 ? 2 : 4;              // code-bit slots the expansion handles
    constexpr int DW = FP4 ? 4 : 2;              // plane dwords per row and stage (128 or 64 depth indices)
    constexpr int PW = 2 * DW;                   // ... and period (two stages)
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN, NT = 64 * WGM * WGN;
    static_assert(BM + BN == NT, "one stacked row per thread");
    static_assert(BM % 64 == 0, "a wavefront's rows belong to one operand");
    constexpr int TILE = NT * DK;                // bytes per stage buffer
    __shared__ __attribute__((aligned(16))) unsigned char lds[4 * TILE];  // two stages being multiplied, two being written
    // STASH (int8 kind, packed-matrix operands): plane words are requested for two periods at a time, 32 adjacent bytes
    // per row and plane; the first period's words go to registers, the second one's straight into this thread's 16-byte
    // places of `raw` (global_load_lds_dwordx4: the 64 lanes' chunks land side by side) and are picked up a period
    // later.  A third fewer requests reach L2; 3 to 9 % faster on four-plane operands, slower for the fp4 kind, whose
    // period already takes 32 adjacent bytes.
    constexpr bool STASH = !CONV && !FP4;
    constexpr int RAWCH = NB * (PW / 4);         // 16-byte chunks per row and period
    __shared__ __attribute__((aligned(16))) unsigned char raw[STASH ? NT * RAWCH * 16 : NT * 4];
    int *const terms = reinterpret_cast<int *>(raw);  // per-row terms of the result (after the loop): W rows, then A rows
    // lowered dword -> (kernel row << 24 | kernel column << 16 | channel word), -1 past the data
    __shared__ __attribute__((aligned(16))) int lut[CONV ? kConvMaxLut + 8 : 4];

    bs::prefetch_kernel_arguments<(int)sizeof(PlanesParams)>();
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int li = lane & 31, lg = lane >> 5;
    int tile_m, tile_n;
    tile_of_workgroup(p.d, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- this thread's row: operand, the plane each code-bit slot takes, masks ----
    const bool isW = tid < BM;
    // Row of the stacked tile this thread owns: within 16 rows, thread bits b3 b2 b1 b0 -> row bits b2 b1 b3 b0, so that
    // the eight lanes an LDS write serves at a time own rows r, r + 1, r + 4, r + 5, r + 8, ...: with the chunk swizzle
    // (row / 4) % 4, which keeps the fragment reads free of bank conflicts, these land in eight different bank groups.
    const int own = (tid & ~15) | ((tid & 6) << 1) | ((tid & 8) >> 2) | (tid & 1);
    const OperandCoding cd = isW ? p.cw : p.ca;
    const int rows = isW ? p.d.M : p.d.N;
    int row = isW ? m0 + own : n0 + (own - BM);
    if (row >= rows) row = rows - 1;             // clamped: its products land in outputs that are never stored
    // CONV, A rows: the row is output pixel (b, oh, ow); pix_h, pix_w = top-left input pixel of its window
    int pix_h = 0, pix_w = 0;
    size_t row_off = (size_t)row * p.Kd;         // dwords from the start of a plane to this row's words
    size_t plane_stride = (size_t)rows * p.Kd;
    if constexpr (CONV) {
        if (!isW) {
            const int b = row / p.cOHW, opix = row - b * p.cOHW;
            const int oh = opix / p.cOW, ow = opix - oh * p.cOW;
            pix_h = oh * p.cStride - p.cPad;
            pix_w = ow * p.cStride - p.cPad;
            row_off = (size_t)b * p.cH * p.cW * p.cPix;            // image b inside a plane
            plane_stride = (size_t)p.cB * p.cH * p.cW * p.cPix;
        }
        for (int q = tid; q < p.Kd + 4; q += NT) {
            const int tap = q / p.cCd, cdw = q - tap * p.cCd;
            const int fr = tap / p.cKW, fs = tap - fr * p.cKW;
            lut[q] = q < p.cKused ? ((fr << 24) | (fs << 16) | cdw) : -1;
        }
        __syncthreads();
    }
    const uint32_t *base = (isW ? p.Wp : p.Ap) + row_off;
    const uint32_t *pl_ptr[NB];
    uint32_t plain[NB], flipped[NB];             // all ones where the slot holds a plane as it is / the inverted top plane
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int pl = q - cd.shift;             // plane of this slot
        const bool has = pl >= 0 && pl < cd.bits;
        pl_ptr[q] = base + (size_t)(has ? pl : 0) * plane_stride;  // an empty slot reads plane 0 and is masked off
        plain[q] = (has && q != cd.top) ? 0xFFFFFFFFu : 0u;
        flipped[q] = (has && q == cd.top) ? 0xFFFFFFFFu : 0u;
        // plain data from here on: x = (r & plain) | (~r & flipped) is one three-input bit operation per word; knowing how
        // the masks came about, the compiler would build selects on their conditions instead
        asm volatile("" : "+v"(plain[q]), "+v"(flipped[q]));
    }
    int popc[NB];                                // popcounts of this row's slots over the depth (for the row-sum terms)
#pragma unroll
    for (int q = 0; q < NB; ++q) popc[q] = 0;
    unsigned char *const my_row = lds + own * DK;
    const int wsw = (own >> 2) & 3;              // chunk swizzle of this row

    // Plane words of one period (two stages) of this row: one request per slot and period where 16 bytes hold both
    // stages (int8 kind), two where they hold one (fp4 kind).  Every lane of a request reads another row, i.e. another
    // cache line, and those line look-ups are what bounds the loader: the fewer requests the better.
    uint32_t R[NB][PW];
    // CONV, A rows: where the four lowered dwords from dword q0 (a multiple of 4) of this row's column lie in an image
    // plane, and which of them exist (taps outside the image and words past the lowered depth read as zero).  The loads
    // themselves are unconditional, from offset 0 where there is nothing to read, and the words are cleared when they
    // are expanded: a load inside a branch would cut the period's instruction stream into pieces and make every wait a
    // wait for all loads.
    int okbits = -1;                             // bit t: word t of R[.] holds data
    auto locate4 = [&](int q0, int (&off)[4]) -> int {
        const int4 l4 = *reinterpret_cast<const int4 *>(&lut[q0]);
        const int l[4] = {l4.x, l4.y, l4.z, l4.w};
        int bits = 0;
#pragma unroll
        for (int t = 0; t < (VEC ? 1 : 4); ++t) {
            const int ih = pix_h + (l[t] >> 24), iw = pix_w + ((l[t] >> 16) & 0xFF);
            const bool ok = l[t] >= 0 && ih >= 0 && ih < p.cH && iw >= 0 && iw < p.cW;
            off[t] = ok ? (ih * p.cW + iw) * p.cPix + (l[t] & 0xFFFF) : 0;
            bits |= ok ? (1 << t) : 0;
        }
        if (VEC) bits = (bits & 1) ? 15 : 0;
        return bits;
    };
    auto gather4 = [&](const uint32_t *img, const int (&off)[4]) -> uint4 {
        if constexpr (VEC) return *reinterpret_cast<const uint4 *>(img + (unsigned)off[0]);
        return make_uint4(img[(unsigned)off[0]], img[(unsigned)off[1]], img[(unsigned)off[2]], img[(unsigned)off[3]]);
    };
    auto fetch = [&](int period) {
        const int s = period < p.nper ? period : p.nper - 1;  // past the depth: any valid address; the words are zeroed on use
        // the second stage of the last period may not exist (the row ends with the first): stay inside the row
        const int o2 = s * PW + 4 < p.Kd ? s * PW + 4 : p.Kd - 4;
        if (CONV && !isW) {                      // uniform for the wavefront
            okbits = 0;
            if constexpr (VEC && PW == 8) {
                // one offset per 16 bytes: both are cheap to keep, and the two requests of a plane, which mostly lie
                // in the same 32 bytes of a pixel's channel run, stay next to each other
                int off0[4], off1[4];
                okbits = locate4(s * PW, off0) | (locate4(o2, off1) << 4);
#pragma unroll
                for (int q = 0; q < NB; ++q) {
                    const uint4 v = gather4(pl_ptr[q], off0), u = gather4(pl_ptr[q], off1);
                    R[q][0] = v.x; R[q][1] = v.y; R[q][2] = v.z; R[q][3] = v.w;
                    R[q][4] = u.x; R[q][5] = u.y; R[q][6] = u.z; R[q][7] = u.w;
                    __builtin_amdgcn_sched_barrier(0);
                }
                return;
            }
#pragma unroll
            for (int g = 0; g < PW / 4; ++g) {   // one gather per 16 bytes of the period's plane words; few offsets live at a time
                int off[4];
                okbits |= locate4(g == 0 ? s * PW : o2, off) << (4 * g);
#pragma unroll
                for (int q = 0; q < NB; ++q) {
                    const uint4 v = gather4(pl_ptr[q], off);
                    R[q][4 * g] = v.x; R[q][4 * g + 1] = v.y; R[q][4 * g + 2] = v.z; R[q][4 * g + 3] = v.w;
                }
            }
            return;
        }
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const uint4 v = *reinterpret_cast<const uint4 *>(pl_ptr[q] + s * PW);
            R[q][0] = v.x; R[q][1] = v.y; R[q][2] = v.z; R[q][3] = v.w;
            if constexpr (PW == 8) {
                const uint4 u = *reinterpret_cast<const uint4 *>(pl_ptr[q] + o2);
                R[q][4] = u.x; R[q][5] = u.y; R[q][6] = u.z; R[q][7] = u.w;
                // the two requests of a row and plane stay next to each other: the second one then finds the first one's
                // line on its way (W2A2 4096^3 49.4 -> 44.1 us; the two-wavefront tile is 3 % faster without)
                if constexpr (NT >= 256) __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // STASH: period -> R as above, period + 1 -> raw (requested next to each other: the two lie in the same 64 bytes
    // of memory, so the second request finds the first one's line on its way)
    lds_void *const raw_wave = (lds_void *)(raw + wave * RAWCH * 1024);
    const unsigned char *const raw_mine = raw + wave * RAWCH * 1024 + lane * 16;
    auto fetch_pair = [&](int period) {
        const int s = period < p.nper ? period : p.nper - 1, s1 = period + 1 < p.nper ? period + 1 : p.nper - 1;
        const int o2 = s * PW + 4 < p.Kd ? s * PW + 4 : p.Kd - 4, o3 = s1 * PW + 4 < p.Kd ? s1 * PW + 4 : p.Kd - 4;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const uint4 v = *reinterpret_cast<const uint4 *>(pl_ptr[q] + s * PW);
            R[q][0] = v.x; R[q][1] = v.y; R[q][2] = v.z; R[q][3] = v.w;
            if constexpr (PW == 8) {
                const uint4 u = *reinterpret_cast<const uint4 *>(pl_ptr[q] + o2);
                R[q][4] = u.x; R[q][5] = u.y; R[q][6] = u.z; R[q][7] = u.w;
            }
            __builtin_amdgcn_global_load_lds((const void *)(pl_ptr[q] + s1 * PW), (lds_void *)((unsigned char __attribute__((address_space(3))) *)raw_wave + q * (PW / 4) * 1024), 16, 0, 0);
            if constexpr (PW == 8)
                __builtin_amdgcn_global_load_lds((const void *)(pl_ptr[q] + o3), (lds_void *)((unsigned char __attribute__((address_space(3))) *)raw_wave + (q * 2 + 1) * 1024), 16, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto unstash = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int q = 0; q < NB; ++q)
#pragma unroll
            for (int h = 0; h < PW / 4; ++h) {
                const uint4 v = *reinterpret_cast<const uint4 *>(raw_mine + (q * (PW / 4) + h) * 1024);
                R[q][4 * h] = v.x; R[q][4 * h + 1] = v.y; R[q][4 * h + 2] = v.z; R[q][4 * h + 3] = v.w;
            }
    };
    // Expands stage `stage` (half `h` of the period in R) and writes its four chunks into stage buffer `buf`.
    // TAIL: the stage may be the last one (an inverted top plane is cut off at the depth) or lie past the depth (the
    // pipeline touches up to three such stages at its end; they become zero codes and stay out of the row sums).
    auto expand_stage = [&](auto tail_c, int buf, int stage, int h) {
        constexpr bool TAIL = decltype(tail_c)::value;
        unsigned char *dst = my_row + buf * TILE;
#pragma unroll
        for (int d = 0; d < DW; ++d) {
            uint32_t vm = 0xFFFFFFFFu, live = 0xFFFFFFFFu;
            if constexpr (TAIL) {
                // validity of the 32 indices of this dword (uniform, scalar arithmetic): ones below the depth
                const int left = p.K32 - 32 * (stage * DW + d);
                vm = left >= 32 ? 0xFFFFFFFFu : (left <= 0 ? 0u : ((1u << left) - 1u));
                live = stage < p.nst ? 0xFFFFFFFFu : 0u;
            }
            uint32_t x[NB];
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                uint32_t r = R[q][h * DW + d];
                if constexpr (CONV) r &= (uint32_t)__builtin_amdgcn_sbfe(okbits, h * DW + d, 1);  // all ones or zero
                x[q] = TAIL ? (((r & plain[q]) | (~r & flipped[q] & vm)) & live) : ((r & plain[q]) | (~r & flipped[q]));
                // one value from here on: left transparent, the two terms are carried through the merges below separately
                // (shifts and masks distribute over the OR) and joined at the end, at 1.6 times the instructions
                asm("" : "+v"(x[q]));
                popc[q] += __builtin_popcount(x[q]);
            }
            if constexpr (FP4) {
                *reinterpret_cast<uint4 *>(dst + 16 * (d ^ wsw)) = expand32_fp4(x[0], x[1]);
            } else {
                uint4 o0, o1;
                expand32_i8(x, o0, o1);
                *reinterpret_cast<uint4 *>(dst + 16 * ((2 * d) ^ wsw)) = o0;
                *reinterpret_cast<uint4 *>(dst + 16 * ((2 * d + 1) ^ wsw)) = o1;
            }
        }
    };

    typename AccOf<FP4>::type acc[WTM][WTN];
#pragma unroll
    for (int a = 0; a < WTM; ++a)
#pragma unroll
        for (int b = 0; b < WTN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    // fragment addresses: row r of the tile, logical chunk c at r * 64 + 16 * (c ^ ((r / 4) % 4))
    const int fsw = (li >> 2) & 3;
    const int rowW = (wm * 32 * WTM + li) * DK, rowA = (BM + wn * 32 * WTN + li) * DK;
    v4i fa[2][WTM], fb[2][WTN];
    auto load_frags = [&](int set, int buf, int sub) {
        const int off = 16 * ((2 * sub + lg) ^ fsw);
        const unsigned char *bw = lds + buf * TILE + rowW + off, *ba = lds + buf * TILE + rowA + off;
#pragma unroll
        for (int a = 0; a < WTM; ++a) fa[set][a] = *reinterpret_cast<const v4i *>(bw + a * 32 * DK);
#pragma unroll
        for (int b = 0; b < WTN; ++b) fb[set][b] = *reinterpret_cast<const v4i *>(ba + b * 32 * DK);
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int a = 0; a < WTM; ++a)
#pragma unroll
            for (int b = 0; b < WTN; ++b) acc[a][b] = mma<FP4>(fa[set][a], fb[set][b], acc[a][b]);
    };
    // spread the other work of a quarter between its matrix instructions: NV vector instructions and one LDS read each
    auto interleave = [&](auto nv_c) {
        constexpr int NV = decltype(nv_c)::value;
#pragma unroll
        for (int r = 0; r < WTM * WTN; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          // MFMA
            if constexpr (NV > 0) __builtin_amdgcn_sched_group_barrier(0x002, NV, 0);   // VALU
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                          // DS read
        }
    };
    constexpr std::integral_constant<int, 0> kNoValu{};
    constexpr std::integral_constant<int, (FP4 ? 60 : 100) / (WTM * WTN) + 1> kExpandValu{};

    // One period = two stages = four depth steps ("quarters").  PP: parity of the period; its stages sit in LDS
    // buffers 2 PP and 2 PP + 1, the next period's stages are written into the other two.  The fragments of a quarter
    // are read during the quarter before.  Quarter 1 expands the next period's first stage, quarter 2 its second one;
    // the barrier behind quarter 2 is the only one of the period: by then every wavefront has written its rows of the
    // next two stages and has received the last fragments of this period (read in quarter 2), so quarter 3 may read the
    // next period's first fragments and request the plane words of the period after next into R, which the two
    // expansions have just released.  TAIL: one of the stages to expand may be the last one or lie past the depth.
    auto request = [&](auto pp_c, int P) {       // plane words of period P + 2 (STASH: of two periods, every other period)
        constexpr int PP = decltype(pp_c)::value;
        if constexpr (!STASH) fetch(P + 2);
        else if constexpr (PP == 0) fetch_pair(P + 2);
        else unstash();
    };
    // LATE = false: the schedule described above.  LATE = true (the second four of eight wavefronts, which share
    // their SIMDs with the first four): the same period with the vector work moved by half a period.  The second
    // stage of the next period is expanded in quarter 0, the words of the period after next are requested in quarter
    // 1, and its first stage is expanded in quarter 3, behind the barrier, into this period's first buffer (nobody
    // reads that one after quarter 0).  The two wavefronts of a SIMD then alternate between a quarter of matrix
    // instructions only and a quarter with the expansion between them, instead of both expanding at the same time:
    // a SIMD does not issue vector and matrix instructions of one wavefront together, but it does overlap one
    // wavefront's matrix instruction with the other's vector instructions.
    auto period = [&](auto pp_c, auto tail_c, auto late_c, int P) __attribute__((always_inline)) {
        constexpr int PP = decltype(pp_c)::value;
        constexpr bool LATE = decltype(late_c)::value;
        constexpr int B0 = 2 * PP, B1 = 2 * PP + 1, N0 = 2 * (PP ^ 1), N1 = 2 * (PP ^ 1) + 1;
        if constexpr (!LATE) {
            load_frags(1, B0, 1);
            mfmas(0);
            interleave(kNoValu);
            __builtin_amdgcn_sched_barrier(0);
            expand_stage(tail_c, N0, 2 * P + 2, 0);
            load_frags(0, B1, 0);
            mfmas(1);
            interleave(kExpandValu);
            __builtin_amdgcn_sched_barrier(0);
            expand_stage(tail_c, N1, 2 * P + 3, 1);
            load_frags(1, B1, 1);
            mfmas(0);
            interleave(kExpandValu);
            __builtin_amdgcn_sched_barrier(0);
            // the smaller tiles request the next words before the barrier, as soon as the registers are free (4 to 5 %
            // faster: the wait at the barrier is time the requests are on their way); the 256 x 256 tile behind it (3 to 5 %
            // slower the other way round)
            if constexpr (NT < 512) {
                request(pp_c, P);
                __builtin_amdgcn_sched_barrier(0);
            }
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (NT == 512) request(pp_c, P);
            load_frags(0, N0, 0);
            mfmas(1);
            interleave(kNoValu);
            __builtin_amdgcn_sched_barrier(0);
        } else {
            expand_stage(tail_c, N1, 2 * P + 3, 1);
            load_frags(1, B0, 1);
            mfmas(0);
            interleave(kExpandValu);
            __builtin_amdgcn_sched_barrier(0);
            request(pp_c, P);
            load_frags(0, B1, 0);
            mfmas(1);
            interleave(kNoValu);
            __builtin_amdgcn_sched_barrier(0);
            load_frags(1, B1, 1);
            mfmas(0);
            interleave(kNoValu);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            expand_stage(tail_c, B0, 2 * P + 4, 0);
            load_frags(0, N0, 0);
            mfmas(1);
            interleave(kExpandValu);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    auto run = [&](auto late_c) __attribute__((always_inline)) {
        constexpr bool LATE = decltype(late_c)::value;
        // prologue: the first period expanded, the second requested (LATE: and its first stage expanded)
        fetch(0);
        expand_stage(std::true_type{}, 0, 0, 0);
        expand_stage(std::true_type{}, 1, 1, 1);
        fetch(1);
        if constexpr (LATE) expand_stage(std::true_type{}, 2, 2, 0);
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        load_frags(0, 0, 0);
        int P = 0;
        for (; 2 * P + 8 <= p.nst; P += 2) {      // the stages expanded here (up to 2 P + 6) lie wholly inside the depth
            period(I0{}, std::false_type{}, late_c, P);
            period(I1{}, std::false_type{}, late_c, P + 1);
        }
        for (; P + 1 < p.nper; P += 2) {
            period(I0{}, std::true_type{}, late_c, P);
            period(I1{}, std::true_type{}, late_c, P + 1);
        }
        if (P < p.nper) period(I0{}, std::true_type{}, late_c, P);
    };
    // every wavefront passes the same number of barriers on either path
    if (NT == 512 && wave >= 4) run(std::true_type{});
    else run(std::false_type{});

    // ---- per-row terms of the affine correction: slot q carries weight 2^(q - shift) of the unsigned code ----
    // They go where the stashed plane words were.  The last periods still request words past the depth (clamped
    // addresses, never read back): those writes into `raw` have to land before the terms do, the first wavefront's
    // places being where every wavefront's terms go.
    if constexpr (STASH) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    {
        int rs = 0;
#pragma unroll
        for (int q = 0; q < NB; ++q) rs = wrap_add(rs, (q - cd.shift >= 0) ? (popc[q] << (q - cd.shift)) : 0);
        terms[own] = isW ? wrap_add(wrap_mul(p.row_coef, rs), p.row_const) : wrap_mul(p.col_coef, rs);
    }
    __syncthreads();
    PlanesResult result{p.mul, p.acc_scale, terms, terms + BM};
    dense_epilogue<WTM, WTN, FUSE, FP4, WGM, WGN>(p.d, acc, lds, m0, n0, tile_m, result);
}

// v = alpha u + beta with u the unsigned code the kernel multiplies
void affine_of(int bits, bs_format fmt, int &alpha, int &beta)
{
    alpha = 1; beta = 0;
    if (fmt == BS_BIPOLAR) { alpha = 2; beta = -1; }
    if (fmt == BS_TWOS_COMPLEMENT) beta = -(1 << (bits - 1));
}

OperandCoding coding_of(int bits, bs_format fmt, bool fp4)
{
    OperandCoding c;
    c.bits = bits;
    c.shift = fp4 ? 2 - bits : 0;
    c.top = fmt == BS_TWOS_COMPLEMENT ? c.shift + bits - 1 : -1;
    return c;
}

template <bool FP4, int WTM, int WTN, int WGM, int WGN>
bs_status launch_tile(PlanesParams &p, bool fuse, bool conv, hipStream_t st)
{
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN, NT = 64 * WGM * WGN;
    p.d.gx = (p.d.N + BN - 1) / BN;
    p.d.gy = (p.d.M + BM - 1) / BM;
    const long long blocks = (long long)p.d.gx * p.d.gy;
    if (blocks >= (1LL << 31)) return BS_ERR_UNSUPPORTED;
    // panels: a tile's rows x the packed depth x the operand's planes; an XCD holds 32, 64 or 128 workgroups of the three tiles
    plan_tile_order(p.d, (long long)BM * p.Kd * 4 * p.cw.bits, (long long)BN * p.Kd * 4 * p.ca.bits, (int)(NT == 512 ? 32 : NT == 256 ? 64 : 128));
    if (conv) {  // implicit lowering exists with the thresholding epilogue only
        if (!fuse) return BS_ERR_UNSUPPORTED;
        if (p.cCd % 4 == 0 && p.cPix % 4 == 0) planes_mfma_kernel<FP4, WTM, WTN, WGM, WGN, true, true, true><<<dim3((unsigned)blocks), NT, 0, st>>>(p);
        else planes_mfma_kernel<FP4, WTM, WTN, WGM, WGN, true, true, false><<<dim3((unsigned)blocks), NT, 0, st>>>(p);
    } else if (fuse) planes_mfma_kernel<FP4, WTM, WTN, WGM, WGN, true><<<dim3((unsigned)blocks), NT, 0, st>>>(p);
    else planes_mfma_kernel<FP4, WTM, WTN, WGM, WGN, false><<<dim3((unsigned)blocks), NT, 0, st>>>(p);
    return bs::after_launch();
}

template <bool FP4>
bs_status launch_kind(PlanesParams &p, bool fuse, bool conv, hipStream_t st)
{
    // 256 x 256 tiles on eight wavefronts (one per compute unit), 128 x 128 on four (two per compute unit) or, for
    // small outputs, 64 x 64 on two (each wavefront 32 x 64).  A smaller tile expands more rows per product, but puts
    // more workgroups on the chip: bs_planes_tile holds the rule, which the engine choice's time model shares.
    int tile = bs_planes_tile(p.d.M, p.d.N, nullptr, nullptr);
    // The implicit-lowering kernels keep their look-up table in LDS as well, so that a compute unit holds three
    // workgroups of the 64 x 64 tile instead of four: beyond 768 tiles these take the larger tile (conv3 of Table 2 at
    // batch 64, 1014 tiles: 27 us instead of 15.6).
    if (conv && tile == 64 && ((p.d.M + 63) / 64) * (long long)((p.d.N + 63) / 64) > 768) tile = 128;
    if (tile == 256) return launch_tile<FP4, 4, 2, 2, 4>(p, fuse, conv, st);
    if (tile == 64) return launch_tile<FP4, 1, 2, 2, 1>(p, fuse, conv, st);
    return launch_tile<FP4, 2, 2, 2, 2>(p, fuse, conv, st);
}

}  // namespace

bool planes_mfma_supported(int wbits, bs_format wfmt, int abits, bs_format afmt, int64_t K, bool fp4)
{
    if (K >= (int64_t(1) << 30)) return false;  // the kernels count depth indices in 32 bits
    if (!fp4) return true;
    if (wbits > 2 || abits > 2) return false;
    // the fp32 sum of products of unsigned codes (in quarter steps) stays exact
    return K * ((int64_t(1) << wbits) - 1) * ((int64_t(1) << abits) - 1) < (int64_t(1) << 24);
}

bs_status launch_planes_mfma(const PlanesGemm &q, bool fp4, bool fuse, hipStream_t st)
{
    if (!planes_mfma_supported(q.wbits, q.wfmt, q.abits, q.afmt, q.K, fp4)) return BS_ERR_UNSUPPORTED;
    PlanesParams p{};
    p.d.M = q.M; p.d.N = q.N;
    p.d.C = q.C; p.d.ldc = q.ldc;
    p.d.thr = q.thr; p.d.obits = q.obits; p.d.T = fuse ? (1 << q.obits) - 1 : 0;
    p.d.Y = q.Y; p.d.Yd = q.Yd;
    p.Wp = q.W; p.Ap = q.A; p.Kd = q.Kd;
    p.cw = coding_of(q.wbits, q.wfmt, fp4);
    p.ca = coding_of(q.abits, q.afmt, fp4);
    p.K32 = (int)q.K;
    int aw, bw, aa, ba;
    affine_of(q.wbits, q.wfmt, aw, bw);
    affine_of(q.abits, q.afmt, aa, ba);
    p.mul = aw * aa;
    p.row_coef = aw * ba;
    p.row_const = (int)((unsigned)(bw * ba) * (unsigned)q.K);   // modulo 2^32, like every sum of terms
    p.col_coef = bw * aa;
    // a 2-bit code in an E2M1 nibble is the number u / 2
    p.acc_scale = fp4 ? (float)((q.wbits == 2 ? 2 : 1) * (q.abits == 2 ? 2 : 1)) : 1.0f;
    const int per_stage = fp4 ? 128 : 64;
    p.nst = (int)((q.K + per_stage - 1) / per_stage);
    p.nper = (p.nst + 1) / 2;
    if (q.conv) {
        if (2 * (int64_t)q.Kd > 2 * kConvMaxLut) return BS_ERR_UNSUPPORTED;
        p.cH = q.cH; p.cW = q.cW; p.cCd = q.cCd; p.cPix = q.cPix; p.cKW = q.cKW; p.cStride = q.cStride; p.cPad = q.cPad;
        p.cOW = q.cOW; p.cOHW = q.cOHW; p.cB = q.cB; p.cKused = q.cKused;
    }
    return fp4 ? launch_kind<true>(p, fuse, q.conv != 0, st) : launch_kind<false>(p, fuse, q.conv != 0, st);
}

}  // namespace bs
