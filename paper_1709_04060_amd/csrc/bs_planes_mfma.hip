// Matrix-core engine on PACKED PLANES: the product W . A of Sec. 3.1 computed with MFMA
// instructions from the same bit-plane operands the AND-popcount kernels take.  This is the
// byte-wise engine of the paper's per-layer choice (Sec. 4.1.1, 4.2) without its cost in memory:
// operands stay w/8 and a/8 byte per element in device memory, nothing unpacked is ever written
// there, and no extra buffer or launch is needed.  The loader of the kernel turns plane bits into
// operand codes on their way to LDS:
//   fp4 kind   operands of at most 2 bits (any format): every value is a number of the 4-bit E2M1
//              floating-point format; v_mfma_f32_32x32x64_f8f6f4, 128 depth indices per 64-byte
//              LDS row and stage, exact while K max|w| max|a| < 2^24;
//   int8 kind  operands of up to 4 bits; v_mfma_i32_32x32x32_i8, 64 depth indices per row and stage.
//
// Expansion.  A thread owns one row of the stacked [W rows; A rows] tile.  For two planes x0, x1 the
// even-indexed bits of both are merged into one word of 2-bit fields (x0 & 0x55..) | (x1 & 0x55..) << 1,
// the odd-indexed ones likewise; a byte of such a word holds four fields, which one byte-permute and one
// packed 16-bit multiply spread to the low bits of four bytes; those bytes index a four-entry code table
// held in a register through one more byte-permute instruction (v_perm_b32).  The table carries the format (unsigned, two's
// complement, bipolar), so one code path serves all of them.  A bipolar operand (value 2 bit - 1) takes
// a synthetic second plane "index < K": padding bits then decode to 0 instead of -1.  Operands with
// fewer planes than the kernel variant handles get their missing planes masked to zero.  Planes 2 and
// 3 (int8 kind) go through a second table holding 4 b2 + 8 b3 (or -8 b3), added byte-wise.
//
// Pipeline.  Two LDS stage buffers of 64-byte rows (XOR-swizzled 16-byte chunks, the layout of the
// direct-to-LDS dense kernel), one barrier per stage in the middle of the stage: the first half of
// iteration i expands the second half of stage i + 1 and multiplies depth step 0 of stage i, the
// second half expands the first half of stage i + 2 and multiplies depth step 1; plane words are
// requested from memory one iteration before they are expanded.  Expansion (VALU) and matrix
// instructions are issued interleaved from the same basic block, so the vector and the matrix
// pipe work at the same time.
#include "bs_dense_common.h"
#include "bs_gemm_kernel.h"

namespace bs {
namespace {

using namespace bs::dense;

struct PlanesParams {
    DenseParams d;          // epilogue fields (M, N, C, ldc, thr, T, obits, Y, Yd, gx, gy); W, A, ld*, K unused
    const uint32_t *Wp;     // [wbits][M][Kd]
    const uint32_t *Ap;     // [abits][N][Kd]
    int Kd;                 // dwords per packed row
    int wbits, abits;
    int wbip, abip;         // operand is bipolar
    int K32;                // depth in indices (below 2^30)
    int nst;                // stages: ceil(K / indices per stage)
    uint32_t lutW[4];       // code tables of the weight operand: fp4 {even nibble, odd nibble}; int8 {planes 0-1, planes 2-3}
    uint32_t lutA[4];
};

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// A word of 2-bit fields (four per byte) split into its even and odd nibbles, one nibble per byte.
struct FieldWord {
    uint32_t lo, hi;  // byte g: fields 0, 1 of byte g of the word | fields 2, 3
};
__device__ __forceinline__ FieldWord split_nibbles(uint32_t c)
{
    FieldWord f;
    f.lo = c & 0x0F0F0F0Fu;
    f.hi = (c >> 4) & 0x0F0F0F0Fu;
    return f;
}

// The four fields of byte g -> the low two bits of four bytes.  A byte-permute puts the byte's low nibble into
// the low half-word and its high nibble into the high half-word; one packed 16-bit multiply by (1 + 2^6) moves
// the second field of each nibble from bits 2-3 to bits 8-9 (its other copies are masked off).
template <int G>
__device__ __forceinline__ uint32_t spread_fields(const FieldWord &f)
{
    const uint32_t in = __builtin_amdgcn_perm(f.hi, f.lo, 0x0c000c00u | (uint32_t)G | ((uint32_t)(4 + G) << 16));
    const u16x2 m = __builtin_bit_cast(u16x2, in) * (u16x2){0x41, 0x41};
    return __builtin_bit_cast(uint32_t, m) & 0x03030303u;
}

// even-indexed and odd-indexed bits of two planes merged into 2-bit fields (plane 0 | plane 1 << 1)
__device__ __forceinline__ void merge_planes(uint32_t x0, uint32_t x1, FieldWord &even, FieldWord &odd)
{
    even = split_nibbles((x0 & 0x55555555u) | ((x1 & 0x55555555u) << 1));
    odd = split_nibbles(((x0 >> 1) & 0x55555555u) | (x1 & 0xAAAAAAAAu));
}

template <int G>
__device__ __forceinline__ uint32_t codes8_fp4(const FieldWord &e, const FieldWord &o, uint32_t lut_lo, uint32_t lut_hi)
{
    return __builtin_amdgcn_perm(0u, lut_lo, spread_fields<G>(e)) | __builtin_amdgcn_perm(0u, lut_hi, spread_fields<G>(o));
}

// 32 depth indices of two planes -> 32 E2M1 codes (16 bytes; low nibble = even index)
__device__ __forceinline__ uint4 expand32_fp4(uint32_t x0, uint32_t x1, uint32_t lut_lo, uint32_t lut_hi)
{
    FieldWord e, o;
    merge_planes(x0, x1, e, o);
    return make_uint4(codes8_fp4<0>(e, o, lut_lo, lut_hi), codes8_fp4<1>(e, o, lut_lo, lut_hi),
                      codes8_fp4<2>(e, o, lut_lo, lut_hi), codes8_fp4<3>(e, o, lut_lo, lut_hi));
}

// eight depth indices of four planes -> eight int8 values (two dwords).  The two tables' bytes add without carries
// between bytes: planes 0-1 give 0..3 whenever planes 2-3 exist.
template <int G>
__device__ __forceinline__ void values8_i8(const FieldWord (&e)[2], const FieldWord (&o)[2], uint32_t lut01, uint32_t lut23,
                                           uint32_t &d0, uint32_t &d1)
{
    const uint32_t ve = __builtin_amdgcn_perm(0u, lut01, spread_fields<G>(e[0])) + __builtin_amdgcn_perm(0u, lut23, spread_fields<G>(e[1]));
    const uint32_t vo = __builtin_amdgcn_perm(0u, lut01, spread_fields<G>(o[0])) + __builtin_amdgcn_perm(0u, lut23, spread_fields<G>(o[1]));
    d0 = __builtin_amdgcn_perm(vo, ve, 0x05010400u);  // e0 o0 e1 o1
    d1 = __builtin_amdgcn_perm(vo, ve, 0x07030602u);  // e2 o2 e3 o3
}

// 32 depth indices of four planes -> 32 int8 values (two 16-byte chunks)
__device__ __forceinline__ void expand32_i8(const uint32_t (&x)[4], uint32_t lut01, uint32_t lut23, uint4 &out0, uint4 &out1)
{
    FieldWord e[2], o[2];
    merge_planes(x[0], x[1], e[0], o[0]);
    merge_planes(x[2], x[3], e[1], o[1]);
    values8_i8<0>(e, o, lut01, lut23, out0.x, out0.y);
    values8_i8<1>(e, o, lut01, lut23, out0.z, out0.w);
    values8_i8<2>(e, o, lut01, lut23, out1.x, out1.y);
    values8_i8<3>(e, o, lut01, lut23, out1.z, out1.w);
}

// FP4: operand kind.  WTM x WTN MFMA tiles of 32 x 32 per wavefront, WGM x WGN wavefronts; the workgroup has as many
// threads as the stacked tile has rows (one row per thread).
template <bool FP4, int WTM, int WTN, int WGM, int WGN, bool FUSE>
__global__ void __launch_bounds__(64 * WGM * WGN)
planes_mfma_kernel(const PlanesParams p)
{
    constexpr int NB = FP4 ? 2 : 4;              // planes the expansion handles
    constexpr int DW = FP4 ? 4 : 2;              // plane dwords per row and stage (128 or 64 depth indices)
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN, NT = 64 * WGM * WGN;
    static_assert(BM + BN == NT, "one stacked row per thread");
    static_assert(BM % 64 == 0, "a wavefront's rows belong to one operand");
    constexpr int TILE = NT * DK;                // bytes per stage buffer
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * TILE];

    bs::prefetch_kernel_arguments<(int)sizeof(PlanesParams)>();
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int li = lane & 31, lg = lane >> 5;
    const int tile_m = blockIdx.x / p.d.gx, tile_n = blockIdx.x % p.d.gx;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- this thread's row: operand, plane pointers, plane masks, code tables ----
    const bool isW = tid < BM;
    const int bits = isW ? p.wbits : p.abits;
    const bool bip = (isW ? p.wbip : p.abip) != 0;
    const int rows = isW ? p.d.M : p.d.N;
    int row = isW ? m0 + tid : n0 + (tid - BM);
    if (row >= rows) row = rows - 1;             // clamped: its products land in outputs that are never stored
    const uint32_t *base = (isW ? p.Wp : p.Ap) + (size_t)row * p.Kd;
    const uint32_t *pl_ptr[NB];
    uint32_t keep[NB];                           // all ones for a plane the operand has
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int qe = q < bits ? q : bits - 1;  // a missing plane reads an existing one (and is masked off)
        pl_ptr[q] = base + (size_t)qe * rows * p.Kd;
        keep[q] = (q < bits) ? 0xFFFFFFFFu : 0u;
    }
    const uint32_t valid_on = bip ? 0xFFFFFFFFu : 0u;  // bipolar: plane 1 := "index < K"
    const uint32_t lutX = isW ? p.lutW[0] : p.lutA[0], lutY = isW ? p.lutW[1] : p.lutA[1];
    unsigned char *const my_row = lds + tid * DK;
    const int wsw = (tid >> 1) & 3;              // chunk swizzle of this row

    uint32_t R[2][NB][DW];
    auto fetch = [&](int set, int stage) {
        const int s = stage < p.nst ? stage : p.nst - 1;  // past the depth: any valid address; the result is never multiplied
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            if constexpr (DW == 4) {
                const uint4 v = *reinterpret_cast<const uint4 *>(pl_ptr[q] + s * 4);
                R[set][q][0] = v.x; R[set][q][1] = v.y; R[set][q][2] = v.z; R[set][q][3] = v.w;
            } else {
                const uint2 v = *reinterpret_cast<const uint2 *>(pl_ptr[q] + s * 2);
                R[set][q][0] = v.x; R[set][q][1] = v.y;
            }
        }
    };
    // Expands plane dword dwi of the stage held in register set `set` and writes its chunks into buffer `buf`.
    auto expand_dword = [&](int set, int buf, int stage, int dwi) {
        uint32_t x[NB];
        x[0] = R[set][0][dwi];                   // every operand has plane 0
#pragma unroll
        for (int q = 1; q < NB; ++q) x[q] = R[set][q][dwi] & keep[q];
        // validity of the 32 indices of this dword (uniform, scalar arithmetic): ones below the depth
        const int left = p.K32 - 32 * (stage * DW + dwi);
        const uint32_t vm = left >= 32 ? 0xFFFFFFFFu : (left <= 0 ? 0u : ((1u << left) - 1u));
        x[1] |= vm & valid_on;
        unsigned char *dst = my_row + buf * TILE;
        if constexpr (FP4) {
            *reinterpret_cast<uint4 *>(dst + 16 * (dwi ^ wsw)) = expand32_fp4(x[0], x[1], lutX, lutY);
        } else {
            uint4 o0, o1;
            expand32_i8(x, lutX, lutY, o0, o1);
            *reinterpret_cast<uint4 *>(dst + 16 * ((2 * dwi) ^ wsw)) = o0;
            *reinterpret_cast<uint4 *>(dst + 16 * ((2 * dwi + 1) ^ wsw)) = o1;
        }
    };
    // half 0: the chunks depth step 0 reads (0, 1); half 1: chunks 2, 3
    auto expand_half = [&](int set, int buf, int stage, int half) {
        if constexpr (FP4) {
            expand_dword(set, buf, stage, 2 * half);
            expand_dword(set, buf, stage, 2 * half + 1);
        } else {
            expand_dword(set, buf, stage, half);
        }
    };

    typename AccOf<FP4>::type acc[WTM][WTN];
#pragma unroll
    for (int a = 0; a < WTM; ++a)
#pragma unroll
        for (int b = 0; b < WTN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    // fragment addresses: row r of the tile, logical chunk c at r * 64 + 16 * (c ^ ((r / 2) % 4))
    const int fsw = (li >> 1) & 3;
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
    // spread the vector work of a half between its matrix instructions
    auto interleave = [&]() {
#pragma unroll
        for (int r = 0; r < WTM * WTN; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          // MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, FP4 ? 150 / (WTM * WTN) + 1 : 140 / (WTM * WTN) + 1, 0);  // VALU
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                          // DS read
        }
    };

    // One iteration = one stage (see the header comment).  PAR: parity of the stage = its LDS buffer and register set.
    auto step = [&](auto par, int i) {
        constexpr int PAR = decltype(par)::value;
        expand_half(PAR ^ 1, PAR ^ 1, i + 1, 1);
        load_frags(1, PAR, 1);
        mfmas(0);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        // every LDS operation of this wavefront is complete (reads of this stage arrived, writes of the next one
        // done) before anybody goes on
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        fetch(PAR ^ 1, i + 3);
        load_frags(0, PAR ^ 1, 0);
        expand_half(PAR, PAR, i + 2, 0);
        mfmas(1);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
    };

    fetch(0, 0);
    fetch(1, 1);
    expand_half(0, 0, 0, 0);
    expand_half(0, 0, 0, 1);
    fetch(0, 2);
    expand_half(1, 1, 1, 0);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    load_frags(0, 0, 0);
    int i = 0;
    for (; i + 1 < p.nst; i += 2) {
        step(std::integral_constant<int, 0>{}, i);
        step(std::integral_constant<int, 1>{}, i + 1);
    }
    if (i < p.nst) step(std::integral_constant<int, 0>{}, i);

    dense_epilogue<WTM, WTN, FUSE, FP4, WGM, WGN>(p.d, acc, lds, m0, n0, tile_m);
}

int fp4_code(int v)
{
    const int mag = v < 0 ? -v : v;
    int code;
    switch (mag) {
    case 0: code = 0x0; break;
    case 1: code = 0x2; break;
    case 2: code = 0x4; break;
    case 3: code = 0x5; break;
    case 4: code = 0x6; break;
    case 6: code = 0x7; break;
    default: return -1;
    }
    return v < 0 ? (code | 0x8) : code;
}

// Value tables of one operand, indexed by the 2-bit field (b_lo | b_hi << 1) of a plane pair.
void value_tables(int bits, bs_format fmt, int (&v01)[4], int (&v23)[4])
{
    int cw[4] = {0, 0, 0, 0};
    for (int i = 0; i < bits; ++i) cw[i] = (fmt == BS_TWOS_COMPLEMENT && i == bits - 1) ? -(1 << i) : (1 << i);
    for (int f = 0; f < 4; ++f) {
        v01[f] = cw[0] * (f & 1) + cw[1] * (f >> 1);
        v23[f] = cw[2] * (f & 1) + cw[3] * (f >> 1);
    }
    if (fmt == BS_BIPOLAR) {  // plane 1 is the synthetic "index < K" plane
        v01[0] = 0; v01[1] = 0; v01[2] = -1; v01[3] = 1;
    }
}

bool fill_tables(int bits, bs_format fmt, bool fp4, uint32_t (&lut)[4])
{
    int v01[4], v23[4];
    value_tables(bits, fmt, v01, v23);
    lut[0] = lut[1] = lut[2] = lut[3] = 0;
    for (int f = 0; f < 4; ++f) {
        if (fp4) {
            const int c = fp4_code(v01[f]);
            if (c < 0 || v23[f] != 0) return false;
            lut[0] |= (uint32_t)c << (8 * f);
            lut[1] |= (uint32_t)(c << 4) << (8 * f);
        } else {
            lut[0] |= (uint32_t)(v01[f] & 0xFF) << (8 * f);
            lut[1] |= (uint32_t)(v23[f] & 0xFF) << (8 * f);
        }
    }
    return true;
}

template <bool FP4, int WTM, int WTN, int WGM, int WGN>
bs_status launch_tile(PlanesParams &p, bool fuse, hipStream_t st)
{
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN, NT = 64 * WGM * WGN;
    p.d.gx = (p.d.N + BN - 1) / BN;
    p.d.gy = (p.d.M + BM - 1) / BM;
    const long long blocks = (long long)p.d.gx * p.d.gy;
    if (blocks >= (1LL << 31)) return BS_ERR_UNSUPPORTED;
    if (fuse) planes_mfma_kernel<FP4, WTM, WTN, WGM, WGN, true><<<dim3((unsigned)blocks), NT, 0, st>>>(p);
    else planes_mfma_kernel<FP4, WTM, WTN, WGM, WGN, false><<<dim3((unsigned)blocks), NT, 0, st>>>(p);
    return bs::after_launch();
}

template <bool FP4>
bs_status launch_kind(PlanesParams &p, bool fuse, hipStream_t st)
{
    // 256 x 256 tiles on eight wavefronts (one per compute unit) or 128 x 128 on four (two or more per compute
    // unit).  A 128 x 128 tile expands half the rows of a 256 x 256 one for a quarter of its products, and the
    // expansion is what bounds the kernel: the small tile is taken when it needs fewer rounds over the chip.
    auto tiles = [&](int b) { return (long long)((p.d.M + b - 1) / b) * ((p.d.N + b - 1) / b); };
    const long long big = (tiles(256) + 255) / 256 * 100, small = (tiles(128) + 511) / 512 * 55;
    if (big <= small) return launch_tile<FP4, 4, 2, 2, 4>(p, fuse, st);
    return launch_tile<FP4, 2, 2, 2, 2>(p, fuse, st);
}

}  // namespace

bool planes_mfma_supported(int wbits, bs_format wfmt, int abits, bs_format afmt, int64_t K, bool fp4)
{
    if (K >= (int64_t(1) << 30)) return false;  // the kernels count depth indices in 32 bits
    if (!fp4) return true;
    if (wbits > 2 || abits > 2) return false;
    return K * max_abs(wbits, wfmt) * max_abs(abits, afmt) < (int64_t(1) << 24);  // fp32 accumulation stays exact
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
    p.wbits = q.wbits; p.abits = q.abits;
    p.wbip = q.wfmt == BS_BIPOLAR; p.abip = q.afmt == BS_BIPOLAR;
    p.K32 = (int)q.K;
    const int per_stage = fp4 ? 128 : 64;
    p.nst = (int)((q.K + per_stage - 1) / per_stage);
    if (!fill_tables(q.wbits, q.wfmt, fp4, p.lutW) || !fill_tables(q.abits, q.afmt, fp4, p.lutA)) return BS_ERR_UNSUPPORTED;
    return fp4 ? launch_kind<true>(p, fuse, st) : launch_kind<false>(p, fuse, st);
}

}  // namespace bs
