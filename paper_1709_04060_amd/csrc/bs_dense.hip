// Dense engine: the product of two few-bit integer matrices (Sec. 3.1 of the paper,
// "W . A") computed on the matrix cores from UNPACKED int8 operands, with the same
// thresholding epilogue (Sec. 2.1.1) as the bit-serial engine.
//
// Why it exists.  The paper chooses per layer between a bit-serial engine and an 8-bit
// engine (Sec. 4.2) and states the break-even rule: bit-serial wins while w * a stays
// below the ratio of binary to 8-bit peak throughput (Sec. 4.1.1).  On gfx950 that ratio
// is below one: one v_and + v_bcnt pair does 32 binary MACs per lane, an int8 MFMA does
// 1024 MACs per cycle and SIMD.  For compute-bound shapes the dense contraction therefore
// belongs on MFMA; bit-serial keeps the bandwidth-bound shapes, where bytes scale with bits.
//
// Kernel shape.  A workgroup of four wavefronts (2 x 2) - eight (2 x 4) for the 256 x 256 tile of
// the direct-to-LDS kernel - owns a BM x BN tile of C; each wavefront owns WTM x WTN tiles of
// 32 x 32 accumulated with v_mfma_i32_32x32x32_i8.
// Operands are depth-contiguous int8 rows; 64 bytes of depth per row and stage are
// fetched global -> registers one stage ahead, then written to LDS with an 80-byte row
// stride so that the 16-byte fragment reads of 32 consecutive rows spread over all banks.
// Both operands give lane l the depth bytes [16 (l / 32), 16 (l / 32) + 16) of row l % 32,
// so the contraction is over matching depth indices whatever order the instruction uses
// internally.  Accumulator register v of lane l is C[8 (v / 4) + 4 (l / 32) + v % 4][l % 32]
// of its 32 x 32 tile.
#include "bs_dense_common.h"

namespace {

using namespace bs::dense;

template <int WTM, int WTN, bool FUSE, bool FP4>
__global__ void __launch_bounds__(256)
dense_gemm_kernel(const DenseParams p)
{
    constexpr int BM = 64 * WTM, BN = 64 * WTN;
    constexpr int ROWS = BM + BN;
    constexpr int CPT = ROWS * DCH / 256;  // chunks each thread moves per stage
    static_assert((ROWS * DCH) % 256 == 0 && (BM * DCH) % 256 == 0, "loader slots are uniform");
    constexpr int TILE_BYTES = ROWS * DROW;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * TILE_BYTES];  // two stages: one read, one written

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lg = lane >> 5;
    int tile_m, tile_n;
    tile_of_workgroup(p, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- loader: thread moves chunk (row, c) of the stacked [W rows; A rows] tile ----
    // Loads are unconditional and never feed anything but the later LDS write, so many can
    // be in flight: rows beyond M / N are clamped to the last row (their products land in
    // outputs that are never stored), chunks beyond the depth are read from the row's first
    // chunk and zeroed when the stage is written to LDS.
    const int8_t *rowp[CPT];
    int lofs[CPT];
#pragma unroll
    for (int s = 0; s < CPT; ++s) {
        const int id = tid + s * 256;
        const int row = id / DCH, c = id % DCH;
        lofs[s] = row * DROW + c * 16;
        if (s * 256 < BM * DCH) {
            const int m = m0 + row < p.M ? m0 + row : p.M - 1;
            rowp[s] = p.W + (long long)m * p.ldw;
        } else {
            const int n = n0 + (row - BM) < p.N ? n0 + (row - BM) : p.N - 1;
            rowp[s] = p.A + (long long)n * p.lda;
        }
    }
    // two stages in flight in registers: enough bytes outstanding to cover memory latency
    uint4 stage[2][CPT];
    auto fetch = [&](int ring, int k0) {
#pragma unroll
        for (int s = 0; s < CPT; ++s) {
            const int k = k0 + ((tid + s * 256) % DCH) * 16;
            stage[ring][s] = *reinterpret_cast<const uint4 *>(rowp[s] + (k < p.K ? k : 0));
        }
    };
    // LDS write of the stage that starts at depth kst.  FULL: the stage lies wholly inside
    // the depth, nothing to mask.
    auto commit = [&](auto full, int ring, int buf, int kst) {
#pragma unroll
        for (int s = 0; s < CPT; ++s) {
            uint4 v = stage[ring][s];
            if constexpr (!decltype(full)::value) {
                const int k = kst + ((tid + s * 256) % DCH) * 16;
                v = k < p.K ? mask_tail(v, k, p.K) : make_uint4(0, 0, 0, 0);
            }
            *reinterpret_cast<uint4 *>(lds + buf * TILE_BYTES + lofs[s]) = v;
        }
    };

    typename AccOf<FP4>::type acc[WTM][WTN];
#pragma unroll
    for (int a = 0; a < WTM; ++a)
#pragma unroll
        for (int b = 0; b < WTN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    const unsigned char *ldsW = lds + (wm * 32 * WTM + li) * DROW + lg * 16;
    const unsigned char *ldsA = lds + (BM + wn * 32 * WTN + li) * DROW + lg * 16;

    // Stage k is consumed from one LDS buffer while stage k + 1 (fetched during the previous
    // iteration) is written to the other and stage k + 2 is requested from memory.  The
    // fragments of the next 32-byte depth step are read from LDS before the MFMAs of the
    // current one are issued, so LDS latency hides behind matrix work; the single barrier of
    // a stage sits between its two depth steps, after which the next stage's buffer is
    // complete and may be read.
    static_assert(DK == 64, "the pipeline below is written for two depth steps per stage");
    v4i fa[2][WTM], fb[2][WTN];
    auto load_frags = [&](int set, int buf, int sub) {
        const unsigned char *bw = ldsW + buf * TILE_BYTES + sub * 32, *ba = ldsA + buf * TILE_BYTES + sub * 32;
#pragma unroll
        for (int a = 0; a < WTM; ++a) fa[set][a] = *reinterpret_cast<const v4i *>(bw + a * 32 * DROW);
#pragma unroll
        for (int b = 0; b < WTN; ++b) fb[set][b] = *reinterpret_cast<const v4i *>(ba + b * 32 * DROW);
    };
    auto mfmas = [&](int set) {
#pragma unroll
        for (int a = 0; a < WTM; ++a)
#pragma unroll
            for (int b = 0; b < WTN; ++b)
                acc[a][b] = mma<FP4>(fa[set][a], fb[set][b], acc[a][b]);
    };

    // One stage of the pipeline.  PAR = parity of the stage index = LDS buffer it is read
    // from; stage k + 1 sits in register ring (PAR ^ 1) and goes to the other LDS buffer,
    // then that ring is refilled with stage k + 3.
    // One stage of the pipeline.  PAR = parity of the stage index = LDS buffer it is read
    // from; stage k + 1 sits in register ring (PAR ^ 1) and goes to the other LDS buffer,
    // then that ring is refilled with stage k + 3.  FAST steps are branch-free (stages k + 1
    // exists and is full), which also lets the compiler count outstanding loads exactly and
    // wait only for the older of the two rings.
    // The scheduling fences keep the order "issue LDS reads, issue all MFMAs of the step,
    // only then wait": left alone, the compiler hoists the barrier (and the wait for the
    // reads just issued) above the MFMAs and the matrix pipe idles during LDS latency.
    const int nst = (p.K + DK - 1) / DK;      // stages
    const int nfull = p.K / DK;               // stages wholly inside the depth
    const int nst_even = (nst + 1) & ~1;      // a surplus stage multiplies zeros
    auto step = [&](auto par, auto fast, int i) {
        constexpr int PAR = decltype(par)::value;
        constexpr bool FAST = decltype(fast)::value;
        const int k0 = i * DK;
        const bool more = FAST || i + 1 < nst_even;
        // first half: write stage k + 1 to LDS, read the fragments of depth step 1, MFMAs of step 0
        if (more) commit(fast, PAR ^ 1, PAR ^ 1, k0 + DK);
        load_frags(1, PAR, 1);
        mfmas(0);
        if constexpr (FAST) {
            // one LDS operation between consecutive MFMAs: the four wavefronts of a workgroup
            // run in lockstep between barriers, so without interleaving they all move data at
            // once and then all multiply at once, and LDS and matrix time add up
#pragma unroll
            for (int r = 0; r < CPT; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // DS write
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();  // stage k + 1 is now complete in the other buffer; nobody reads this one's step 0 any more
        // second half: request stage k + 3, read the next stage's first fragments, MFMAs of step 1
        if (more) {
            fetch(PAR ^ 1, k0 + 3 * DK);
            load_frags(0, PAR ^ 1, 0);
        }
        mfmas(1);
        if constexpr (FAST) {
#pragma unroll
            for (int r = 0; r < CPT; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    fetch(0, 0);
    commit(std::false_type{}, 0, 0, 0);
    fetch(1, DK);
    fetch(0, 2 * DK);
    __syncthreads();
    load_frags(0, 0, 0);
    int i = 0;
    for (; i + 2 < nfull; i += 2) {           // stages i + 1 and i + 2 are full
        step(P0{}, std::true_type{}, i);
        step(P1{}, std::true_type{}, i + 1);
    }
    for (; i < nst_even; i += 2) {
        step(P0{}, std::false_type{}, i);
        step(P1{}, std::false_type{}, i + 1);
    }

    dense_epilogue<WTM, WTN, FUSE, FP4>(p, acc, lds, m0, n0, tile_m);
}

// ------------------------------------------------------------------ variant with direct global -> LDS loads
// Same tiling and MFMA schedule; the operand stages go from memory straight into LDS
// (global_load_lds_dwordx4), three stages deep, without passing through registers: no
// ds_write instructions, no staging registers, loads issued a stage and a half ahead of
// their use.  Such a load writes the 64 lanes' 16 bytes to consecutive LDS addresses, so
// a row is 64 unpadded bytes; bank conflicts of the fragment reads are avoided by an XOR
// swizzle applied on the GLOBAL side (lane l of a load fetches chunk (l % 4) ^ f(row) of
// its row, f(row) = (row / 4) % 4: measured with a read-only probe, 16-byte fragment reads of 32 rows of 64 bytes
// take 3.4 ns per wavefront read with this function or with rows padded to 80 bytes, 3.9 ns with (row / 2) % 4,
// 7.0 ns with row % 4 or without a swizzle) and undone by the reader.  Needs a depth of whole 16-byte
// chunks (a last stage of fewer than four chunks is completed with zeros written by the lanes
// that have nothing to load); other depths use the register-staged kernel above.
typedef __attribute__((address_space(3))) void lds_void;

template <int WTM, int WTN, bool FUSE, bool FP4, int WGM = 2, int WGN = 2>
__global__ void __launch_bounds__(64 * WGM * WGN)
dense_gemm_lds_kernel(const DenseParams p)
{
    constexpr int NBUF = 3;                      // stage i + NBUF - 1 is requested while stage i is consumed (4 measured: no gain)
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN;
    constexpr int ROWS = BM + BN;
    constexpr int TILE = ROWS * DK;              // bytes per stage, rows unpadded
    constexpr int LPW = ROWS / 16 / (WGM * WGN); // load instructions per wavefront and stage (16 rows each)
    static_assert(ROWS % (16 * WGM * WGN) == 0, "every wavefront issues the same number of loads");
    __shared__ __attribute__((aligned(16))) unsigned char lds[NBUF * TILE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int li = lane & 31, lg = lane >> 5;
    int tile_m, tile_n;
    tile_of_workgroup(p, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- loader: instruction j of this wavefront covers stacked rows (wave * LPW + j) * 16 .. + 15 ----
    const int8_t *gsrc[LPW];
    int gchunk[LPW];  // byte offset of this lane's chunk within a stage's 64 depth bytes
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
        const int row = (wave * LPW + j) * 16 + (lane >> 2);
        const int c = (lane & 3) ^ ((row >> 2) & 3);
        gchunk[j] = c * 16;
        if (row < BM) {
            const int m = m0 + row < p.M ? m0 + row : p.M - 1;
            gsrc[j] = p.W + (long long)m * p.ldw + c * 16;
        } else {
            const int n = n0 + (row - BM) < p.N ? n0 + (row - BM) : p.N - 1;
            gsrc[j] = p.A + (long long)n * p.lda + c * 16;
        }
    }
    auto issue = [&](int buf, int k0) {
#pragma unroll
        for (int j = 0; j < LPW; ++j)
            __builtin_amdgcn_global_load_lds((const void *)(gsrc[j] + k0), (lds_void *)(lds + buf * TILE + (wave * LPW + j) * 16 * DK),
                                             16, 0, 0);
    };
    // The last stage of a depth that is a multiple of 16 but not of 64 bytes: lanes whose chunk lies past the
    // depth write zeros instead of loading.  The first chunk of every row is inside the depth, so each of
    // the LPW load instructions still has active lanes and the load counter advances as for a full stage.
    auto issue_tail = [&](int buf, int k0) {
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            unsigned char *dst = lds + buf * TILE + (wave * LPW + j) * 16 * DK;
            if (k0 + gchunk[j] < p.K)
                __builtin_amdgcn_global_load_lds((const void *)(gsrc[j] + k0), (lds_void *)dst, 16, 0, 0);
            else
                *reinterpret_cast<uint4 *>(dst + lane * 16) = make_uint4(0, 0, 0, 0);
        }
    };

    typename AccOf<FP4>::type acc[WTM][WTN];
#pragma unroll
    for (int a = 0; a < WTM; ++a)
#pragma unroll
        for (int b = 0; b < WTN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0;

    // fragment addresses: row r of the tile, logical chunk c -> r * 64 + 16 * (c ^ f(r)); the
    // tile rows of a lane differ by multiples of 32, so f(r) = (li / 4) % 4 for all of them
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
            for (int b = 0; b < WTN; ++b)
                acc[a][b] = mma<FP4>(fa[set][a], fb[set][b], acc[a][b]);
    };

    const int nfull = p.K / DK, nst = (p.K + DK - 1) / DK;  // whole stages, and stages with the partial last one
    // One stage.  MODE 1: stage i + 2 exists and is requested now (branch-free main loop, so that
    // the loads can be spread between the MFMAs); MODE 2: the same for the partial last stage;
    // MODE 0: the last two stages run without requests.
    auto step = [&](auto mode_t, int i, int cur) {
        constexpr int MODE = decltype(mode_t)::value;
        constexpr bool MORE = MODE != 0;
        const int nxt = cur == NBUF - 1 ? 0 : cur + 1, last = cur == 0 ? NBUF - 1 : cur - 1;
        // buffer `last` held stage i - 1: nobody reads it after the previous iteration's barrier
        if constexpr (MODE == 1) issue(last, (i + NBUF - 1) * DK);
        if constexpr (MODE == 2) issue_tail(last, (i + NBUF - 1) * DK);
        load_frags(1, cur, 1);
        mfmas(0);
        if constexpr (MORE) {
#pragma unroll
            for (int r = 0; r < LPW; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // VMEM read (the LDS-bound loads)
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // A bare s_barrier with explicit counters: __syncthreads() carries a full fence, i.e. a
        // wait for ALL outstanding loads, including the ones issued for later stages.  Needed
        // here: this wavefront's part of stage i + 1 has landed (the (NBUF - 2) * LPW newer loads
        // may stay outstanding) and its LDS reads of the current buffer are done.
        if constexpr (MORE) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((NBUF - 2) * LPW) : "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        if (MORE || i + 1 < nst) load_frags(0, nxt, 0);
        mfmas(1);
#pragma unroll
        for (int r = 0; r < LPW; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue: stages 0 .. NBUF - 2 requested, stage 0 awaited
#pragma unroll
    for (int st = 0; st < NBUF - 1; ++st) {
        if (st < nfull) issue(st, st * DK);
        else if (st < nst) issue_tail(st, st * DK);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    load_frags(0, 0, 0);
    int cur = 0, i = 0;
    for (; i + NBUF - 1 < nfull; ++i) {
        step(std::integral_constant<int, 1>{}, i, cur);
        cur = cur == NBUF - 1 ? 0 : cur + 1;
    }
    if (i + NBUF - 1 < nst) {  // the partial last stage is requested here (at most once)
        step(std::integral_constant<int, 2>{}, i, cur);
        cur = cur == NBUF - 1 ? 0 : cur + 1;
        ++i;
    }
    for (; i < nst; ++i) {
        step(std::integral_constant<int, 0>{}, i, cur);
        cur = cur == NBUF - 1 ? 0 : cur + 1;
    }

    dense_epilogue<WTM, WTN, FUSE, FP4, WGM, WGN>(p, acc, lds, m0, n0, tile_m);
}

// ------------------------------------------------------------------ unpack (planes -> int8)
// One thread turns one 32-bit word per plane (32 depth indices of one row) into 32 int8 values.
// Four elements at a time: a nibble of a plane becomes four 0/1 bytes with one multiply
// (n * 0x00204081 puts bit i of n at bit 8 i; the four shifted copies do not overlap), the planes
// add up byte-wise without carries (codes stay below 16), and the sign is filled in with bit
// operations (two's complement: the bits above the code, where the top plane is set; bipolar
// 2 b - 1: 0xFF ^ 0xFE b).
template <int FMT>
__global__ void __launch_bounds__(256)
unpack_kernel(const uint32_t *__restrict__ planes, int bits, long long rows, long long depth, int Kd,
              int8_t *__restrict__ dst, long long ld, long long words_per_row)
{
    const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
    if (item >= rows * words_per_row) return;
    const long long r = item / words_per_row, dw = item - r * words_per_row;
    uint32_t x[4] = {0, 0, 0, 0};
#pragma unroll
    for (int pl = 0; pl < 4; ++pl)
        if (pl < bits) x[pl] = planes[((long long)pl * rows + r) * Kd + dw];
    const uint32_t sign_fill = 0x100u - (1u << bits);  // the byte's bits above a bits-wide code
    uint32_t out[8];
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        uint32_t sp[4];
#pragma unroll
        for (int pl = 0; pl < 4; ++pl) sp[pl] = (((x[pl] >> (4 * g)) & 0xFu) * 0x00204081u) & 0x01010101u;
        uint32_t v;
        if (FMT == BS_BIPOLAR) {
            v = 0xFFFFFFFFu ^ (sp[0] * 0xFEu);
        } else {
            v = sp[0] + 2 * sp[1] + 4 * sp[2] + 8 * sp[3];
            if (FMT == BS_TWOS_COMPLEMENT) {
                const uint32_t top = bits == 1 ? sp[0] : bits == 2 ? sp[1] : bits == 3 ? sp[2] : sp[3];
                v |= top * sign_fill;
            }
        }
        const long long e0 = dw * 32 + 4 * g;  // elements past the depth read as 0 (matters for bipolar: code 0 is -1)
        if (e0 + 4 > depth) v = e0 >= depth ? 0u : v & ((1u << (8 * (int)(depth - e0))) - 1u);
        out[g] = v;
    }
    int8_t *o = dst + r * ld + dw * 32;
    *reinterpret_cast<uint4 *>(o) = make_uint4(out[0], out[1], out[2], out[3]);
    if (dw * 32 + 16 < ((depth + 15) / 16) * 16) *reinterpret_cast<uint4 *>(o + 16) = make_uint4(out[4], out[5], out[6], out[7]);
}

// Tile shapes: WTM x WTN MFMA tiles per wavefront, WGM x WGN wavefronts per workgroup.
template <int WTM, int WTN, int WGM, int WGN, bool FP4>
bs_status launch_dense(DenseParams &p, bool fuse, hipStream_t st)
{
    constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN, NT = 64 * WGM * WGN;
    p.gx = (p.N + BN - 1) / BN;
    p.gy = (p.M + BM - 1) / BM;
    const long long blocks = (long long)p.gx * p.gy;
    if (blocks >= (1LL << 31)) return BS_ERR_UNSUPPORTED;
    // panels: a tile's rows x the depth in bytes; an XCD's 32 compute units hold one workgroup of eight wavefronts
    // (or of four of 64 x 64) each, two of the others
    plan_tile_order(p, (long long)BM * p.K, (long long)BN * p.K, (NT == 512 || (WTM == 4 && WTN == 4)) ? 32 : 64);
    // four wavefronts of 128 x 128 exist in the register-staged kernel only (the direct-to-LDS kernel runs that tile on eight)
    constexpr bool DIRECT = !(WTM == 4 && WTN == 4);
    if (p.K % 16 == 0) {  // whole 16-byte chunks: operands can go straight from memory to LDS
        if constexpr (DIRECT) {
            if (fuse) dense_gemm_lds_kernel<WTM, WTN, true, FP4, WGM, WGN><<<dim3((unsigned)blocks), NT, 0, st>>>(p);
            else dense_gemm_lds_kernel<WTM, WTN, false, FP4, WGM, WGN><<<dim3((unsigned)blocks), NT, 0, st>>>(p);
            return bs::after_launch();
        }
    }
    if constexpr (WGM == 2 && WGN == 2) {  // the register-staged kernel is written for four wavefronts
        if (fuse) dense_gemm_kernel<WTM, WTN, true, FP4><<<dim3((unsigned)blocks), 256, 0, st>>>(p);
        else dense_gemm_kernel<WTM, WTN, false, FP4><<<dim3((unsigned)blocks), 256, 0, st>>>(p);
        return bs::after_launch();
    }
    return BS_ERR_UNSUPPORTED;
}

// Largest tile that still gives every compute unit a workgroup.  With the direct-to-LDS kernel the two large tiles
// run on eight wavefronts (two per SIMD: while one waits at the stage barrier or for its fragments the other keeps
// the matrix pipe busy; 8192^3 int8: 559 -> 452 us, 8192 x 8192 x 1024: 104 -> 83 us); depths with a tail use the
// register-staged kernel and its four-wavefront tiles.
template <bool FP4>
bs_status choose_tile(DenseParams &p, bool fuse, hipStream_t st)
{
    auto tiles = [&](int bm, int bn) { return (long long)((p.M + bm - 1) / bm) * ((p.N + bn - 1) / bn); };
    if (p.K % 16 == 0) {
        // Time ~ rounds over the 256 compute units x time of one round.  Measured round times relative to the
        // 256 x 256 tile (fused epilogue, depths 2304..8192, 18 shapes from 64 to 186624 columns): 128 x 256
        // 0.60, 128 x 128 0.36 (two of its workgroups share a compute unit); on a tie the larger tile.
        auto rounds = [&](int bm, int bn) { return (tiles(bm, bn) + 255) / 256; };
        const long long ca = rounds(256, 256) * 100, cb = rounds(128, 256) * 60, cc = rounds(128, 128) * 36;
        if (ca <= cb && ca <= cc) return launch_dense<4, 2, 2, 4, FP4>(p, fuse, st);
        if (cb <= cc) return launch_dense<2, 2, 2, 4, FP4>(p, fuse, st);
        // 128 x 128 on eight wavefronts of 32 x 64 as well: 10 % faster than on four of 64 x 64 (fp4, fused,
        // 384 x 2304 x 10816: 12.5 vs 14.0 us; 2048^3: 9.1 vs 10.6 us)
        return launch_dense<1, 2, 4, 2, FP4>(p, fuse, st);
    }
    if (tiles(256, 256) >= 256) return launch_dense<4, 4, 2, 2, FP4>(p, fuse, st);
    return launch_dense<2, 2, 2, 2, FP4>(p, fuse, st);
}

// K counts depth indices; the operands hold one (int8) or half a (fp4) byte per index.
template <bool FP4>
bs_status dense_common(const void *W, int64_t ldw, const void *At, int64_t lda, int64_t M, int64_t N, int64_t K,
                       int32_t *C, int64_t ldc, const int32_t *thr, int obits, uint64_t *Yp, bool fuse, void *stream)
{
    const int64_t Kbytes = FP4 ? (K + 1) / 2 : K;
    if (!W || !At || M <= 0 || N <= 0 || K <= 0 || ldw < Kbytes || lda < Kbytes) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(W, 16) || !bs::aligned(At, 16) || (ldw & 15) || (lda & 15)) return BS_ERR_ALIGNMENT;
    if (fuse) {
        if (!thr || !Yp || obits < 1) return BS_ERR_INVALID_ARG;
        if (obits > bs::kMaxBits) return BS_ERR_UNSUPPORTED;
        if (!bs::aligned(thr, 4) || !bs::aligned(Yp, 16)) return BS_ERR_ALIGNMENT;
    } else {
        if (!C || ldc < N) return BS_ERR_INVALID_ARG;
        if (!bs::aligned(C, 4)) return BS_ERR_ALIGNMENT;
    }
    // int8: |w|, |a| <= 128, every partial sum stays below 2^31 while K < 2^17.
    // fp4: |w|, |a| <= 6, every partial sum stays below 2^24 (exact in fp32) while K < 2^18.
    if (K >= (int64_t(1) << (FP4 ? 18 : 17))) return BS_ERR_OVERFLOW_RISK;
    if (M >= (int64_t(1) << 31) || N >= (int64_t(1) << 31)) return BS_ERR_OVERFLOW_RISK;
    DenseParams p;
    p.W = static_cast<const int8_t *>(W); p.A = static_cast<const int8_t *>(At); p.ldw = ldw; p.lda = lda;
    p.M = (int)M; p.N = (int)N; p.K = (int)Kbytes;
    p.C = C; p.ldc = ldc;
    p.thr = thr; p.obits = obits; p.T = fuse ? (1 << obits) - 1 : 0;
    p.Y = reinterpret_cast<uint32_t *>(Yp);
    p.Yd = (int)(2 * bs_words_per_row(M));
    hipStream_t st = static_cast<hipStream_t>(stream);
    return choose_tile<FP4>(p, fuse, st);
}

// ------------------------------------------------------------------ unpack (planes -> fp4 codes)
// One thread turns one 32-bit word per plane (32 depth indices of one row) into 32 E2M1 codes
// (16 bytes, low nibble = even index).  Eight indices at a time: the even bits of a plane byte
// are spread to the low bits of four bytes (a 24-bit multiply and a mask), the planes are
// stacked into a table index per byte, and one byte-permute instruction looks all four up in
// the eight-entry code table (lut_lo: code of index c in byte c); the odd bits go through a
// second table that holds the codes already shifted to the high nibble (lut_hi).
template <int BITS>
__global__ void __launch_bounds__(256)
unpack_fp4_kernel(const uint32_t *__restrict__ planes, uint2 lut_lo, uint2 lut_hi, unsigned rows, long long depth,
                  int Kd, uint8_t *__restrict__ dst, long long ld, unsigned words_per_row)
{
    const unsigned item = blockIdx.x * 256u + threadIdx.x;
    if (item >= rows * words_per_row) return;
    const unsigned r = item / words_per_row, dw = item - r * words_per_row;
    uint32_t x[BITS];
#pragma unroll
    for (int pl = 0; pl < BITS; ++pl) x[pl] = planes[((size_t)pl * rows + r) * Kd + dw];
    const long long left = depth - (long long)dw * 32;  // indices of this word inside the depth (>= 1)
    uint32_t out[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        uint32_t se = 0, so = 0;
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) {
            const uint32_t b = (x[pl] >> (8 * g)) & 0xFFu;
            se |= (__umul24(b & 0x55u, 0x041041u) & 0x01010101u) << pl;
            so |= (__umul24((b >> 1) & 0x55u, 0x041041u) & 0x01010101u) << pl;
        }
        uint32_t o = __builtin_amdgcn_perm(lut_lo.y, lut_lo.x, se) | __builtin_amdgcn_perm(lut_hi.y, lut_hi.x, so);
        const long long n = left - 8 * g;                // +0.0 past the depth
        if (n < 8) o = n <= 0 ? 0u : (o & ((1u << (4 * (int)n)) - 1u));
        out[g] = o;
    }
    *reinterpret_cast<uint4 *>(dst + (size_t)r * ld + (size_t)dw * 16) = make_uint4(out[0], out[1], out[2], out[3]);
}

// E2M1 code of a small integer, -1 if it is not representable (the format holds 0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives)
int fp4_code_of(int v)
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
    return v < 0 ? code | 0x8 : code;
}

}  // namespace

extern "C" bs_status bs_unpack_planes(const uint64_t *planes, int bits, bs_format fmt, int64_t rows, int64_t depth,
                                      int8_t *dst, int64_t ld, void *stream)
{
    if (!planes || !dst || rows <= 0 || depth <= 0) return BS_ERR_INVALID_ARG;
    if (bs_status s = bs::check_bits_fmt(bits, fmt)) return s;
    const int64_t chunks = (depth + 15) / 16;
    if (ld < chunks * 16) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(planes, 16) || !bs::aligned(dst, 16) || (ld & 15)) return BS_ERR_ALIGNMENT;
    const int64_t S = bs_words_per_row(depth);
    if (rows * S * 2 * bits >= (int64_t(1) << 31)) return BS_ERR_OVERFLOW_RISK;
    const int64_t words = (depth + 31) / 32, items = rows * words;
    const dim3 grid((unsigned)((items + 255) / 256));
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t *pw = reinterpret_cast<const uint32_t *>(planes);
    if (fmt == BS_BIPOLAR) unpack_kernel<BS_BIPOLAR><<<grid, 256, 0, st>>>(pw, bits, rows, depth, (int)(2 * S), dst, ld, words);
    else if (fmt == BS_TWOS_COMPLEMENT)
        unpack_kernel<BS_TWOS_COMPLEMENT><<<grid, 256, 0, st>>>(pw, bits, rows, depth, (int)(2 * S), dst, ld, words);
    else unpack_kernel<BS_UNSIGNED><<<grid, 256, 0, st>>>(pw, bits, rows, depth, (int)(2 * S), dst, ld, words);
    return bs::after_launch();
}

extern "C" bs_status bs_gemm_i8(const int8_t *W, int64_t ldw, const int8_t *At, int64_t lda, int64_t M, int64_t N,
                                int64_t K, int32_t *C, int64_t ldc, void *stream)
{
    return dense_common<false>(W, ldw, At, lda, M, N, K, C, ldc, nullptr, 0, nullptr, false, stream);
}

extern "C" bs_status bs_gemm_i8_threshold(const int8_t *W, int64_t ldw, const int8_t *At, int64_t lda, int64_t M,
                                          int64_t N, int64_t K, const int32_t *thr, int obits, uint64_t *Yp,
                                          void *stream)
{
    return dense_common<false>(W, ldw, At, lda, M, N, K, nullptr, 0, thr, obits, Yp, true, stream);
}

extern "C" bs_status bs_unpack_planes_fp4(const uint64_t *planes, int bits, bs_format fmt, int64_t rows, int64_t depth,
                                          uint8_t *dst, int64_t ld, void *stream)
{
    if (!planes || !dst || rows <= 0 || depth <= 0) return BS_ERR_INVALID_ARG;
    if (bs_status s = bs::check_bits_fmt(bits, fmt)) return s;
    const int64_t words = (depth + 31) / 32;
    if (ld < words * 16) return BS_ERR_INVALID_ARG;
    if (!bs::aligned(planes, 16) || !bs::aligned(dst, 16) || (ld & 15)) return BS_ERR_ALIGNMENT;
    const int64_t S = bs_words_per_row(depth);
    if (rows * S * 2 * bits >= (int64_t(1) << 31)) return BS_ERR_OVERFLOW_RISK;
    unsigned long long lut = 0;
    for (int c = 0; c < (1 << bits); ++c) {
        int v = c;
        if (fmt == BS_BIPOLAR) v = 2 * c - 1;
        else if (fmt == BS_TWOS_COMPLEMENT && c >= (1 << (bits - 1))) v = c - (1 << bits);
        const int code = fp4_code_of(v);
        if (code < 0) return BS_ERR_UNSUPPORTED;  // 3-bit unsigned (5, 7) and every 4-bit format
        lut |= (unsigned long long)code << (4 * c);
    }
    uint32_t lo[2] = {0, 0}, hi[2] = {0, 0};  // byte c: the code of index c, and the same code in the high nibble
    for (int c = 0; c < (1 << bits); ++c) {
        const uint32_t code = (uint32_t)(lut >> (4 * c)) & 0xFu;
        lo[c / 4] |= code << (8 * (c % 4));
        hi[c / 4] |= (code << 4) << (8 * (c % 4));
    }
    const int64_t items = rows * words;
    const dim3 grid((unsigned)((items + 255) / 256));
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint32_t *pw = reinterpret_cast<const uint32_t *>(planes);
    const uint2 l2 = make_uint2(lo[0], lo[1]), h2 = make_uint2(hi[0], hi[1]);
    if (bits == 1) unpack_fp4_kernel<1><<<grid, 256, 0, st>>>(pw, l2, h2, (unsigned)rows, depth, (int)(2 * S), dst, ld, (unsigned)words);
    else if (bits == 2) unpack_fp4_kernel<2><<<grid, 256, 0, st>>>(pw, l2, h2, (unsigned)rows, depth, (int)(2 * S), dst, ld, (unsigned)words);
    else unpack_fp4_kernel<3><<<grid, 256, 0, st>>>(pw, l2, h2, (unsigned)rows, depth, (int)(2 * S), dst, ld, (unsigned)words);
    return bs::after_launch();
}

extern "C" bs_status bs_gemm_fp4(const uint8_t *W, int64_t ldw, const uint8_t *At, int64_t lda, int64_t M, int64_t N,
                                 int64_t K, int32_t *C, int64_t ldc, void *stream)
{
    return dense_common<true>(W, ldw, At, lda, M, N, K, C, ldc, nullptr, 0, nullptr, false, stream);
}

extern "C" bs_status bs_gemm_fp4_threshold(const uint8_t *W, int64_t ldw, const uint8_t *At, int64_t lda, int64_t M,
                                           int64_t N, int64_t K, const int32_t *thr, int obits, uint64_t *Yp,
                                           void *stream)
{
    return dense_common<true>(W, ldw, At, lda, M, N, K, nullptr, 0, thr, obits, Yp, true, stream);
}
