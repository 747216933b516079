// Bit-serial GEMM (Alg. 2 built from the AND-popcount BinaryGEMM of Alg. 1), with the
// plane-pair weighting and, optionally, successive thresholding (Sec. 2.1.1) fused
// into the epilogue.
//
// General form.  With packed bits Wb[i], Ab[j] the logical operands are
//   W = sum_i cw_i Wb[i] + ow,   A = sum_j ca_j Ab[j] + oa
// (unsigned: cw_i = 2^i; two's complement: top plane negated, the sign rule of Alg. 2;
// bipolar: value = 2 bit - 1, i.e. cw_0 = 2, ow = -1).  Then
//   C[m][n] = sum_ij cw_i ca_j P_ij[m][n] + ow sum_j ca_j popA_j[n]
//             + oa sum_i cw_i popW_i[m] + ow oa K,
//   P_ij[m][n] = sum_d popcount(Wb[i][m][d] & Ab[j][n][d])      (Alg. 1)
// where popW / popA are row popcounts of the planes.  Padding bits are zero in both
// operands, so all counts run over the true depth.
//
// Kernel shape (CDNA4): a workgroup owns a BM x BN tile of C and walks the depth in
// stages of 32 dwords (1024 bits) per packed row.  Each stage is fetched from global
// memory into registers while the previous one is being consumed, then written to LDS
// as 16-byte chunks, XOR-swizzled so that the eight distinct rows a ds_read_b128
// touches fall in eight different bank groups.  A wavefront is an 8 x 8 grid of lanes,
// each lane holding a TM x TN block of int32 accumulators; per 16-byte chunk it reads
// TM weight rows and TN activation columns per plane from LDS and issues
// v_and_b32 + v_bcnt_u32_b32 (whose add operand makes the accumulation free), in the
// AND / popcount / idle-slot rhythm that lets the two wavefronts of a SIMD interleave
// (see mac_block).
// Small output grids use 32 x 32 tiles whose four wavefronts split each stage's depth
// among themselves (KS = 4) and add their partial sums in LDS, so that enough
// wavefronts exist to fill 1024 SIMDs.
//
// Workgroups are dealt round-robin to the chip's 8 XCDs, each with its own L2.  For
// large grids the linear workgroup index is therefore mapped so that every XCD owns one
// compact rectangle of the tile grid and pulls only that rectangle's weight rows and
// activation columns through its L2.
#pragma once
#include "bs_common.h"
#include <type_traits>

namespace bs {

constexpr int kStageDwords = 32;  // dwords of depth per packed row and stage
constexpr long long kIdleMinBlocks = 257;  // more workgroups than compute units (measured: 10.9 vs 12.5 us at 320, 10.7 vs 9.6 us at 256)

// Division of a 32-bit index by a launch constant as a multiply-high and two shifts (the set-up of
// a workgroup is a single wavefront's serial code, where a plain division costs about forty
// instructions and there are up to nine of them).  Exact for every 32-bit numerator.
struct FastDiv {
    uint32_t mul;
    int sh1, sh2;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    int l = 0;
    while ((1ull << l) < d) ++l;  // ceil(log2 d)
    FastDiv f;
    f.mul = (uint32_t)((((1ull << l) - d) << 32) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l > 1 ? l - 1 : 0;
    return f;
}
__device__ __forceinline__ int fdiv(int n, const FastDiv &f)
{
    const uint32_t t = __umulhi(f.mul, (uint32_t)n);
    return (int)((t + (((uint32_t)n - t) >> f.sh1)) >> f.sh2);
}

struct GemmParams {
    const uint32_t *W;  // dword view of Wp
    const uint32_t *A;  // dword view of Ap
    int M, N;
    int Kd;             // dwords per packed row (2 * S)
    int coef[16];       // cw_i * ca_j at [i * 4 + j]
    int crow[4];        // oa * cw_i   (row-popcount correction weights)
    int ccol[4];        // ow * ca_j   (column-popcount correction weights)
    int c0;             // ow * oa * K
    int32_t *C;
    long long ldc;
    const int32_t *thr; // [M][T]
    int T, obits;
    uint32_t *Y;        // dword view of Yp
    int Yd;             // dwords per column of Yp (2 * S_M)
    // tile grid and its mapping onto the linear workgroup index (see tile_of_block)
    int gx, gy;         // tiles along N and along M
    int rx, ry;         // XCD regions along N and M (rx * ry == 8), or 0 = plain row-major order
    int hx, hy;         // tiles per region along N and M
    // implicit lowering (CONV kernels): A points at packed HWC image planes
    int cH, cW;         // image size
    int cCd;            // 32-bit words copied per pixel and tap, ceil(C / 32)
    int cPix;           // 32-bit words between pixels
    int cKW;            // kernel width (taps per kernel row)
    int cStride, cPad;
    int cOW;            // output width
    int cOHW;           // output pixels per image (columns n = (b * cOHW) + oh * cOW + ow)
    int cB;             // images in the batch
    int cKused;         // dwords of a lowered column that carry data: kh * kw * cCd
    int cVec;           // 1 if cCd and cPix are multiples of 4: a 16-byte chunk never straddles two taps
    // max pooling folded into the implicit lowering (pK > 0): A points at the UNPOOLED planes [abits][cB][pH][pW][cPix]
    // and cH x cW is the pooled map the convolution reads, cH = (pH - pK) / pS + 1
    int pK, pS;         // pooling window (at most 3) and stride
    int pH, pW;         // size of the unpooled map
    // single-column kernel: read the weights with the non-temporal hint (set for large weight sets)
    int stream_weights;
    // divisors of the workgroups' set-up code (filled by finish_params)
    FastDiv dGx, dHx, dRx, dT, dOHW, dOW, dCd, dKW;
};

// to be called once the fields above are final, before the launch
inline void finish_params(GemmParams &g)
{
    auto fd = [](int d) { return make_fastdiv(d > 0 ? (uint32_t)d : 1u); };
    g.dGx = fd(g.gx); g.dHx = fd(g.hx); g.dRx = fd(g.rx); g.dT = fd(g.T);
    g.dOHW = fd(g.cOHW); g.dOW = fd(g.cOW); g.dCd = fd(g.cCd); g.dKW = fd(g.cKW);
}

// weight bytes from which the few-column kernel streams past the caches
constexpr long long kStreamWeightBytes = 64ll << 20;

constexpr int kConvMaxLut = 2048;  // lowered dwords the implicit-lowering kernels can index (65536 depth bits)

// GEMV path (bs_gemv_kernel.h, bs_gemv.hip): a workgroup handles at most kGemvMaxCols columns, activation planes in LDS; up to
// kGemvMaxGroupedCols columns run as groups of four side by side (each group streams the weights again, from
// L2 as the groups run together): 32 x 32 tiles would leave 3/4 or more of their columns empty there
// (W4A4 8192 x 8192: 89 us tiled for 5..32 columns, 36 / 53 / 67 us grouped for 8 / 12 / 16).  Between 5 and
// kGemvMaxGroupedCols columns the faster of the two kernels is taken under a time model (gemv_applicable).
constexpr int kGemvMaxCols = 4;
constexpr int kGemvMaxGroupedCols = 16;
constexpr size_t kGemvMaxLds = 64 * 1024;
bool gemv_applicable(const GemmParams &g, int wbits, int abits, bool a_bipolar, bool w_bipolar);
bs_status launch_gemv(const GemmParams &g, int wbits, int abits, bool fuse, bool xr, hipStream_t st);

// Matrix-core engine on packed planes (bs_planes_mfma.hip): the same product from the same operands, plane bits
// expanded to int8 or 4-bit floating-point codes inside the kernel's loader.
struct PlanesGemm {
    const uint32_t *W, *A;  // dword views of the packed operands
    int wbits, abits;
    bs_format wfmt, afmt;
    int M, N;
    int64_t K;
    int Kd;                 // dwords per packed row
    int32_t *C;
    long long ldc;
    const int32_t *thr;
    int obits;
    uint32_t *Y;
    int Yd;
    // implicit lowering (conv != 0): A points at packed HWC image planes [abits][B][H][W][cPix dwords] and column n of
    // the lowered matrix (Sec. 3.2) is gathered from them; fields as in GemmParams
    int conv;
    int cH, cW, cCd, cPix, cKW, cStride, cPad, cOW, cOHW, cB, cKused;
};
bool planes_mfma_supported(int wbits, bs_format wfmt, int abits, bs_format afmt, int64_t K, bool fp4);
bs_status launch_planes_mfma(const PlanesGemm &q, bool fp4, bool fuse, hipStream_t st);

// acc + popcount(x) in ONE instruction: v_bcnt_u32_b32 adds its second operand for
// free.  Written as inline assembly because the optimiser otherwise re-associates a sum
// of popcounts into a tree and pays separate adds for it (25 % more VALU work in the
// inner loop).  Not volatile: the scheduler may move and interleave it freely.
__device__ __forceinline__ int bcnt_acc(uint32_t x, int acc)
{
    int r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
    return r;
}

// Max pooling inside an operand fetch.  Thresholding is monotone, so the maximum of the thresholded codes is the
// thresholded maximum; codes are unsigned and held bit-sliced (one 32-channel word per plane), and the maximum of
// two such numbers is a most-significant-plane-first comparison in bitwise logic.
// pool_load: the channel word at dword offset `at` of the window's top-left pixel, all AB planes, for the 3 x 3 taps a
// window can have.  Every load is unconditional and differs from its neighbours by a wavefront-uniform offset: taps
// beyond a smaller window repeat tap (0, 0), which leaves a maximum unchanged, and an item that is to read as zero
// (padding, past the depth) loads the first words of the map and is cleared by pool_max's `keep` mask.
// V: uint32_t (one 32-channel word) or pool_v4 (a 16-byte chunk of four such words, where a chunk never straddles taps).
typedef unsigned pool_v4 __attribute__((ext_vector_type(4)));
typedef unsigned pool_v2 __attribute__((ext_vector_type(2)));
template <int AB, typename V>
__device__ __forceinline__ void pool_load(const uint32_t *src, int plane_stride, int at, int row_stride, int pix_stride,
                                          int k, bool valid, V (&raw)[9][AB])
{
    if (__builtin_amdgcn_ballot_w64(valid) == 0) {  // nothing to read in this wavefront: no load instructions at all
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int j = 0; j < AB; ++j) raw[t][j] = V(0u);
        return;
    }
    const unsigned lane_off = valid ? (unsigned)at : 0u;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            const int off = (a < k ? a : 0) * row_stride + (b < k ? b : 0) * pix_stride;  // uniform
#pragma unroll
            for (int j = 0; j < AB; ++j) raw[a * 3 + b][j] = *reinterpret_cast<const V *>(src + (j * plane_stride + off) + lane_off);
        }
}
template <int AB, typename V>
__device__ __forceinline__ void pool_max(const V (&raw)[9][AB], uint32_t keep, V (&best)[AB])
{
#pragma unroll
    for (int j = 0; j < AB; ++j) best[j] = raw[0][j];
#pragma unroll
    for (int t = 1; t < 9; ++t) {
        V gt = V(0u), eq = V(0xFFFFFFFFu);  // per channel: raw[t] > best, decided at the highest differing plane
#pragma unroll
        for (int j = AB - 1; j >= 0; --j) {
            gt |= eq & raw[t][j] & ~best[j];
            eq &= ~(raw[t][j] ^ best[j]);
        }
#pragma unroll
        for (int j = 0; j < AB; ++j) best[j] = (gt & raw[t][j]) | (~gt & best[j]);
    }
#pragma unroll
    for (int j = 0; j < AB; ++j) best[j] &= V(keep);
}

// Alg. 1's inner statement on one 16-byte chunk: acc += popcount(a & b) over 4 dwords.
__device__ __forceinline__ int popc_and4(const uint4 &a, const uint4 &b, int acc)
{
    acc = bcnt_acc(a.x & b.x, acc);
    acc = bcnt_acc(a.y & b.y, acc);
    acc = bcnt_acc(a.z & b.z, acc);
    acc = bcnt_acc(a.w & b.w, acc);
    return acc;
}

// The XNOR-popcount binary dot product of prior work (Sec. 3.1) in its XOR form: for +-1
// operands dot = K - 2 popcount(a ^ b); zero padding bits agree in both operands.
__device__ __forceinline__ int popc_xor4(const uint4 &a, const uint4 &b, int acc)
{
    acc = bcnt_acc(a.x ^ b.x, acc);
    acc = bcnt_acc(a.y ^ b.y, acc);
    acc = bcnt_acc(a.z ^ b.z, acc);
    acc = bcnt_acc(a.w ^ b.w, acc);
    return acc;
}

__device__ __forceinline__ uint32_t dword_of(const uint4 &v, int d) { return d == 0 ? v.x : d == 1 ? v.y : d == 2 ? v.z : v.w; }

// Alg. 1's inner statement for a lane's TM x TN outputs on one 16-byte chunk of TM weight rows and TN
// activation columns, as one chain of two-instruction steps: the AND (or XOR) of the next product, then
// the popcount-accumulate of the current one.
//
// The order decides the speed.  A SIMD of this chip executes the AND in two cycles and the popcount in
// four, but one wavefront issues at most one instruction per four cycles, so a lone wavefront needs 8
// cycles per product.  Every step reads the register its predecessor wrote from inside an asm
// statement; for that the compiler leaves one idle issue slot (s_nop 0) between the steps, and in that
// rhythm - AND, popcount, idle - the two resident wavefronts of a SIMD interleave, the AND of one in
// the shadow of the other's popcount: about 6.9 cycles per product measured instead of 8.  Spelling the
// idle slot out inside the statements, or making the popcount depend on the AND directly before it, was
// measured slower (the compiler then adds slots of its own, or the rhythm breaks at statement edges).
template <bool XOR, bool IDLE, int TM, int TN>
__device__ __forceinline__ void mac_block(const uint4 (&w)[TM], const uint4 (&a)[TN], int (&acc)[TM][TN])
{
    if constexpr (!IDLE) {
        // A wavefront alone on its SIMD has nobody to interleave with: plain AND + popcount pairs,
        // 8 cycles per product instead of the 12 the idle slot would make it.
#pragma unroll
        for (int r = 0; r < TM; ++r)
#pragma unroll
            for (int c = 0; c < TN; ++c) acc[r][c] = XOR ? popc_xor4(w[r], a[c], acc[r][c]) : popc_and4(w[r], a[c], acc[r][c]);
        return;
    }
    constexpr int NP = 4 * TM * TN;  // products, dword-major: an accumulator returns every TM * TN steps
    auto wd = [&](int n) { return dword_of(w[(n / TN) % TM], n / (TM * TN)); };
    auto ad = [&](int n) { return dword_of(a[n % TN], n / (TM * TN)); };
    uint32_t t = XOR ? (wd(0) ^ ad(0)) : (wd(0) & ad(0));
#pragma unroll
    for (int n = 0; n < NP; ++n) {
        int &o = acc[(n / TN) % TM][n % TN];
        if (n + 1 < NP) {
            uint32_t tn;
            if constexpr (XOR)
                asm("v_xor_b32 %0, %3, %4\n\tv_bcnt_u32_b32 %1, %2, %1" : "=&v"(tn), "+v"(o) : "v"(t), "v"(wd(n + 1)), "v"(ad(n + 1)));
            else
                asm("v_and_b32 %0, %3, %4\n\tv_bcnt_u32_b32 %1, %2, %1" : "=&v"(tn), "+v"(o) : "v"(t), "v"(wd(n + 1)), "v"(ad(n + 1)));
            t = tn;
        } else {
            asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(o) : "v"(t));
        }
    }
}

// Sums of plane-pair terms are taken modulo 2^32: a partial sum may leave the int32 range although the result
// (bounded by K max|w| max|a| < 2^31, checked on the host) does not, and unsigned arithmetic makes that well defined.
__device__ __forceinline__ int wrap_add(int a, int b) { return (int)((unsigned)a + (unsigned)b); }
__device__ __forceinline__ int wrap_mul(int a, int b) { return (int)((unsigned)a * (unsigned)b); }

__device__ __forceinline__ int popc4(const uint4 &a)
{
    return __builtin_popcount(a.x) + __builtin_popcount(a.y) + __builtin_popcount(a.z) + __builtin_popcount(a.w);
}

// Tile owned by workgroup `bid`.  Returns false for the (few) surplus workgroups of
// the XCD-aware layout.
__device__ __forceinline__ bool tile_of_block(const GemmParams &p, int bid, int &tm, int &tn)
{
    if (p.rx == 0) {
        tm = fdiv(bid, p.dGx);
        tn = bid - tm * p.gx;
        return true;
    }
    const int xcd = bid & 7, local = bid >> 3;
    const int ry = fdiv(xcd, p.dRx), rx = xcd - ry * p.rx;
    const int ly = fdiv(local, p.dHx), lx = local - ly * p.hx;
    tm = ry * p.hy + ly;
    tn = rx * p.hx + lx;
    return ly < p.hy && tm < p.gy && tn < p.gx;
}

// WB, AB: weight / activation planes.  TM x TN: accumulators per lane.  WM x WN:
// wavefronts across the tile, KS: wavefronts across the depth of each stage.  FUSE:
// thresholding epilogue instead of the int32 store.  CORR: popcount correction terms
// needed (some operand is bipolar).
// CONV: the activation operand is not a packed matrix but packed HWC image planes; the
// loader gathers each lowered column's words from the image (Sec. 3.2's lowering folded
// into the operand fetch, so the lowered matrix never exists in memory).
// XOR: both operands bipolar (W1A1): popcount(XOR) instead of popcount(AND), no correction terms.
// KT: dwords of depth per packed row and stage (a multiple of 32; 32 everywhere except the
// 32 x 32 tiles of more than four plane pairs, which take 64: see launch_planes).
// POOL (with CONV): the image the columns are gathered from is the maximum over pK x pK windows of the map in
// memory: every thread forms a few 32-channel words of the pooled, lowered tile per stage (all planes at once, the
// comparison needs them all) instead of copying 16-byte chunks, so that a pooling layer between two convolutions
// costs no launch and its output never exists in memory.
template <int WB, int AB, int TM, int TN, int WM, int WN, int KS, int KT, bool FUSE, bool CORR, bool CONV = false,
          bool XOR = false, bool IDLE = true, bool POOL = false>
__global__ void __launch_bounds__(WM * WN * KS * 64)
bs_gemm_kernel(const GemmParams p)
{
    constexpr int KCH = KT / 4;  // 16-byte chunks per row and stage
    static_assert(!XOR || (WB == 1 && AB == 1 && !CORR), "the XOR form exists for one plane per operand only");
    static_assert(!POOL || CONV, "pooling is part of the implicit lowering");
    constexpr int BM = 8 * TM * WM, BN = 8 * TN * WN, NT = 64 * WM * WN * KS;
    constexpr int WROWS = WB * BM, AROWS = AB * BN, ROWS = WROWS + AROWS;
    constexpr int CHUNKS = ROWS * KCH;
    constexpr int CPT = (CHUNKS + NT - 1) / NT;  // chunks each thread moves per stage
    constexpr int PAIRS = WB * AB;
    constexpr bool PER_PAIR = PAIRS <= 4;        // one accumulator set per plane pair
    constexpr int NACC = PER_PAIR ? PAIRS : 1;
    static_assert(KCH % KS == 0, "the depth split must divide the chunks of a stage");
    static_assert((WROWS * KCH) % NT == 0, "every loader slot is wholly weights or wholly activations");
    static_assert((KS > 1 ? 5 : 1) * BM * BN <= CHUNKS * 16, "epilogue staging must fit in the tile space");

    __shared__ uint4 lds[CHUNKS];
    __shared__ int corr_row[CORR ? BM : 1];
    __shared__ int corr_col[CORR ? BN : 1];
    // lowered dword -> (kernel row, kernel column, channel word), -1 past the data; 16-byte reads
    __shared__ __attribute__((aligned(16))) int lut[CONV ? kConvMaxLut + 4 : 4];
    __shared__ int thr_s[FUSE ? BM * 15 : 1];    // thresholds of the tile's rows, fetched while the first stage is in flight

    prefetch_kernel_arguments<(int)sizeof(GemmParams)>();
    int tile_m, tile_n;
    if (!tile_of_block(p, blockIdx.x, tile_m, tile_n)) return;  // uniform for the workgroup

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int ly = lane >> 3, lx = lane & 7;
    const int ks = wave / (WM * WN), wq = wave % (WM * WN);
    const int wm = wq / WN, wn = wq % WN;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // ---- loader set-up: which chunk of which stacked row this thread moves ----
    int goff[CPT];    // dword offset into W or A of the chunk at stage 0, -1 if out of range
    int loff[CPT];    // destination chunk index in LDS
    int cweight[CPT]; // correction weight of the plane the chunk belongs to
    int cnt[CPT];
    int pix_h[CONV ? CPT : 1], pix_w[CONV ? CPT : 1];  // CONV: top-left input pixel of the column's window
#pragma unroll
    for (int s = 0; s < CPT; ++s) {
        const int id = tid + s * NT;
        const int srow = id / KCH, c = id % KCH;
        goff[s] = -1; loff[s] = 0; cweight[s] = 0; cnt[s] = 0;
        if (CONV) { pix_h[s] = 0; pix_w[s] = 0; }
        if (id < CHUNKS) {
            if (s * NT < WROWS * KCH) {
                const int pl = srow / BM, r = srow % BM;
                loff[s] = srow * KCH + (c ^ ((r / TM) & 7));
                if (m0 + r < p.M) goff[s] = (pl * p.M + m0 + r) * p.Kd + c * 4;
                if (CORR) cweight[s] = p.crow[pl];
            } else {
                const int q = srow - WROWS;
                const int pl = q / BN, r = q % BN;
                loff[s] = srow * KCH + (c ^ ((r / TN) & 7));
                if (n0 + r < p.N) {
                    if constexpr (CONV) {
                        const int b = fdiv(n0 + r, p.dOHW), opix = (n0 + r) - b * p.cOHW;
                        const int oh = fdiv(opix, p.dOW), ow = opix - oh * p.cOW;
                        pix_h[s] = oh * p.cStride - p.cPad;
                        pix_w[s] = ow * p.cStride - p.cPad;
                        goff[s] = (pl * p.cB + b) * p.cH * p.cW * p.cPix;  // base of image b in plane pl
                    } else {
                        goff[s] = (pl * p.N + n0 + r) * p.Kd + c * 4;
                    }
                }
                if (CORR) cweight[s] = p.ccol[pl];
            }
        }
    }
    // POOL: the words of the pooled activation tile this thread forms per stage (dword q of column r)
    constexpr int PITEMS = BN * KT, PPT = POOL ? (PITEMS + NT - 1) / NT : 1;
    int pl_src[PPT], pl_h[PPT], pl_w[PPT], pl_dst[PPT], pl_cnt[PPT];
    uint32_t praw[PPT][9][AB], pkeep[PPT];
    if constexpr (POOL) {
#pragma unroll
        for (int t = 0; t < PPT; ++t) {
            const int u = tid + t * NT, r = u / KT, q = u % KT;
            pl_src[t] = -1; pl_h[t] = 0; pl_w[t] = 0; pl_cnt[t] = 0;
            pl_dst[t] = ((WROWS + r) * KCH + ((q >> 2) ^ ((r / TN) & 7))) * 4 + (q & 3);
            if (u < PITEMS && n0 + r < p.N) {
                const int b = fdiv(n0 + r, p.dOHW), opix = (n0 + r) - b * p.cOHW;
                const int oh = fdiv(opix, p.dOW), ow = opix - oh * p.cOW;
                pl_h[t] = oh * p.cStride - p.cPad;
                pl_w[t] = ow * p.cStride - p.cPad;
                pl_src[t] = b * p.pH * p.pW * p.cPix;  // image b in plane 0 of the unpooled map
            }
        }
    }
    // (Item u is word u % KT of column u / KT.  Columns fastest instead, so that in a partly filled last stage whole
    // wavefronts have nothing to read and skip their loads, measured slower: conv3 behind pool2 8.0 instead of 7.2 us.)
    auto pool_fetch = [&](int k0) {
        const int plane_stride = p.cB * p.pH * p.pW * p.cPix;
#pragma unroll
        for (int t = 0; t < PPT; ++t) {
            const int u = tid + t * NT, l = k0 + u % KT;
            int tap = -1;
            if (u < PITEMS && pl_src[t] >= 0 && l < p.Kd) tap = lut[l];
            const int ih = pl_h[t] + (tap >> 24), iw = pl_w[t] + ((tap >> 16) & 0xFF);  // pixel of the pooled map
            const bool ok = tap >= 0 && ih >= 0 && ih < p.cH && iw >= 0 && iw < p.cW;
            const int at = pl_src[t] + (ih * p.pS * p.pW + iw * p.pS) * p.cPix + (tap & 0xFFFF);
            pool_load<AB, uint32_t>(p.A, plane_stride, at, p.pW * p.cPix, p.cPix, p.pK, ok, praw[t]);
            pkeep[t] = ok ? 0xFFFFFFFFu : 0u;
        }
    };
    auto pool_write = [&]() {
        uint32_t *ldsD = reinterpret_cast<uint32_t *>(lds);
#pragma unroll
        for (int t = 0; t < PPT; ++t) {
            if (tid + t * NT >= PITEMS) continue;
            uint32_t best[AB];
            pool_max<AB, uint32_t>(praw[t], pkeep[t], best);
#pragma unroll
            for (int j = 0; j < AB; ++j) {
                ldsD[pl_dst[t] + j * BN * KCH * 4] = best[j];
                if (CORR) pl_cnt[t] += p.ccol[j] * __popc(best[j]);
            }
        }
    };
    uint4 stage[CPT];
    // DO_W / DO_A: the weight slots, the activation slots or (in the depth loop) both
    auto fetch_part = [&](int k0, auto w_c, auto a_c) {
        constexpr bool DO_W = decltype(w_c)::value, DO_A = decltype(a_c)::value;
        // CONV: the table entries of all activation chunks first (one 16-byte LDS read each),
        // so that a single wait precedes the gathers instead of one per word
        int4 tap4[CONV ? CPT : 1];
        if constexpr (POOL && DO_A) pool_fetch(k0);
        if constexpr (CONV && DO_A && !POOL) {
#pragma unroll
            for (int s = 0; s < CPT; ++s) {
                const int c = (tid + s * NT) % KCH;
                tap4[s] = make_int4(-1, -1, -1, -1);
                if (s * NT >= WROWS * KCH && goff[s] >= 0 && k0 + c * 4 < p.Kd)
                    tap4[s] = *reinterpret_cast<const int4 *>(&lut[k0 + c * 4]);
            }
        }
#pragma unroll
        for (int s = 0; s < CPT; ++s) {
            const int c = (tid + s * NT) % KCH;
            if ((s * NT < WROWS * KCH) ? !DO_W : (!DO_A || POOL)) continue;  // resolved at compile time
            uint4 v = make_uint4(0, 0, 0, 0);
            // Rows of a packed matrix are loaded without a branch: a row past the operand or a chunk past the depth reads
            // the operand's first words instead.  Such rows only feed outputs that are never stored, such chunks are
            // never multiplied (the last, partial stage stops at the depth) and are left out of the popcounts below.
            const bool in_range = goff[s] >= 0 && k0 + c * 4 < p.Kd;
            if (s * NT < WROWS * KCH) {
                // (the kernels that gather lowered columns keep the branch for the weights as well: their small grids
                // measured 0.2 us slower per layer without it, the large plain products 1 to 2 % faster)
                if constexpr (!CONV) v = *reinterpret_cast<const uint4 *>(p.W + (size_t)(unsigned)(in_range ? goff[s] + k0 : 0));
                else if (in_range) v = *reinterpret_cast<const uint4 *>(p.W + (size_t)(unsigned)goff[s] + k0);
            } else if constexpr (!CONV) {
                v = *reinterpret_cast<const uint4 *>(p.A + (size_t)(unsigned)(in_range ? goff[s] + k0 : 0));
            } else {
                if (p.cVec) {
                    // the chunk lies inside one tap of one pixel: one test, one 16-byte load
                    const int l0 = tap4[s].x;
                    const int ih = pix_h[s] + (l0 >> 24), iw = pix_w[s] + ((l0 >> 16) & 0xFF);
                    if (l0 >= 0 && ih >= 0 && ih < p.cH && iw >= 0 && iw < p.cW)
                        v = *reinterpret_cast<const uint4 *>(p.A + (size_t)(unsigned)goff[s] +
                                                             (size_t)(ih * p.cW + iw) * p.cPix + (l0 & 0xFFFF));
                } else {
                    const int l[4] = {tap4[s].x, tap4[s].y, tap4[s].z, tap4[s].w};
                    uint32_t e[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        e[t] = 0;
                        const int ih = pix_h[s] + (l[t] >> 24), iw = pix_w[s] + ((l[t] >> 16) & 0xFF);
                        if (l[t] >= 0 && ih >= 0 && ih < p.cH && iw >= 0 && iw < p.cW)
                            e[t] = p.A[(size_t)(unsigned)goff[s] + (size_t)(ih * p.cW + iw) * p.cPix + (l[t] & 0xFFFF)];
                    }
                    v = make_uint4(e[0], e[1], e[2], e[3]);
                }
            }
            stage[s] = v;
        }
    };
    auto fetch = [&](int k0) { fetch_part(k0, std::true_type{}, std::true_type{}); };

    int acc[NACC][TM][TN];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int r = 0; r < TM; ++r)
#pragma unroll
            for (int c = 0; c < TN; ++c) acc[a][r][c] = 0;

    const int wrow0 = (wm * 8 + ly) * TM;          // first weight row of this lane in the tile
    const int acol0 = (wn * 8 + lx) * TN;          // first activation column
    const uint4 *ldsW = lds + wrow0 * KCH;
    const uint4 *ldsA = lds + (WROWS + acol0) * KCH;

    // The weights of the first stage are requested before the correction counters are cleared and the lowering
    // table is built, so that this set-up runs under their memory latency; the gathers need the table.
    fetch_part(0, std::true_type{}, std::false_type{});
    if (CORR) {
        for (int i = tid; i < BM; i += NT) corr_row[i] = 0;
        for (int i = tid; i < BN; i += NT) corr_col[i] = 0;
    }
    if constexpr (CONV) {
        for (int q = tid; q < p.Kd; q += NT) {
            const int tap = fdiv(q, p.dCd), cd = q - tap * p.cCd;
            const int fr = fdiv(tap, p.dKW), fs = tap - fr * p.cKW;
            lut[q] = q < p.cKused ? ((fr << 24) | (fs << 16) | cd) : -1;
        }
        // a barrier that waits for the table's LDS writes only: __syncthreads() would also wait for the weight
        // loads just requested
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }

    fetch_part(0, std::false_type{}, std::true_type{});
    if constexpr (FUSE) {
        // ride on the first stage's memory latency instead of paying a round trip in the epilogue
        for (int i = tid; i < BM * p.T; i += NT) {
            const int r = fdiv(i, p.dT);
            thr_s[i] = (m0 + r < p.M) ? p.thr[(long long)(m0 + r) * p.T + (i - r * p.T)] : 0x7fffffff;
        }
    }
    // One stage: registers -> LDS, start the next stage's loads, then the products.
    // FULL stages run the chunk loop unrolled; the last stage of a depth that is no
    // multiple of the stage holds zero-filled chunks past the depth and runs, after
    // the loop, a rolled copy that stops at the depth (nq chunks hold data).
    auto run_stage = [&](const int k0, auto full_c) {
        constexpr bool FULL = decltype(full_c)::value;
        const int nq = FULL ? KCH : (p.Kd - k0 + 3) >> 2;
        __syncthreads();  // everyone is done reading the previous stage
#pragma unroll
        for (int s = 0; s < CPT; ++s) {
            if (POOL && s * NT >= WROWS * KCH) continue;  // the activation tile comes from pool_write
            if (tid + s * NT < CHUNKS) lds[loff[s]] = stage[s];
            if constexpr (CORR && CONV) cnt[s] += popc4(stage[s]);  // loaded under a branch: zero where there is nothing
            else if constexpr (CORR) cnt[s] += (goff[s] >= 0 && k0 + ((tid + s * NT) % KCH) * 4 < p.Kd) ? popc4(stage[s]) : 0;
        }
        if constexpr (POOL) pool_write();
        __syncthreads();
        if (FULL && k0 + KT < p.Kd) fetch(k0 + KT);

        if constexpr (PER_PAIR) {
            auto chunk = [&](const int q) {
                uint4 w[WB][TM], a[AB][TN];
#pragma unroll
                for (int i = 0; i < WB; ++i)
#pragma unroll
                    for (int r = 0; r < TM; ++r) w[i][r] = ldsW[(i * BM + r) * KCH + (q ^ ly)];
#pragma unroll
                for (int j = 0; j < AB; ++j)
#pragma unroll
                    for (int c = 0; c < TN; ++c) a[j][c] = ldsA[(j * BN + c) * KCH + (q ^ lx)];
#pragma unroll
                for (int i = 0; i < WB; ++i)
#pragma unroll
                    for (int j = 0; j < AB; ++j) mac_block<XOR, IDLE, TM, TN>(w[i], a[j], acc[i * AB + j]);
            };
            if constexpr (FULL) {
#pragma unroll
                for (int qq = 0; qq < KCH / KS; ++qq) chunk(qq * KS + ks);
            } else {
#pragma unroll 1
                for (int q = ks; q < nq; q += KS) chunk(q);
            }
        } else {
            // Many plane pairs: one pair at a time over the whole stage into a small
            // counter (at most 1024 per stage), then one weighted add per pair and stage.
#pragma unroll 1
            for (int i = 0; i < WB; ++i) {
#pragma unroll 1
                for (int j = 0; j < AB; ++j) {
                    if (p.coef[i * 4 + j] == 0) continue;  // plane pair left out (approximate mode): no work spent on it
                    int t[TM][TN];
#pragma unroll
                    for (int r = 0; r < TM; ++r)
#pragma unroll
                        for (int c = 0; c < TN; ++c) t[r][c] = 0;
                    auto chunk = [&](const int q) {
                        uint4 w[TM], a[TN];
#pragma unroll
                        for (int r = 0; r < TM; ++r) w[r] = ldsW[(i * BM + r) * KCH + (q ^ ly)];
#pragma unroll
                        for (int c = 0; c < TN; ++c) a[c] = ldsA[(j * BN + c) * KCH + (q ^ lx)];
                        mac_block<false, IDLE, TM, TN>(w, a, t);
                    };
                    if constexpr (FULL) {
#pragma unroll
                        for (int qq = 0; qq < KCH / KS; ++qq) chunk(qq * KS + ks);
                    } else {
#pragma unroll 1
                        for (int q = ks; q < nq; q += KS) chunk(q);
                    }
                    const int cf = p.coef[i * 4 + j];
#pragma unroll
                    for (int r = 0; r < TM; ++r)
#pragma unroll
                        for (int c = 0; c < TN; ++c) acc[0][r][c] = wrap_add(acc[0][r][c], __mul24(t[r][c], cf));
                }
            }
        }
    };
    const int Kfull = p.Kd - p.Kd % KT;
    for (int k0 = 0; k0 < Kfull; k0 += KT) run_stage(k0, std::true_type{});
    if (Kfull < p.Kd) run_stage(Kfull, std::false_type{});

    // ---- correction terms (bipolar operands): weighted row popcounts via LDS atomics ----
    if (CORR) {
#pragma unroll
        for (int s = 0; s < CPT; ++s) {
            const int id = tid + s * NT;
            if (id < CHUNKS && cweight[s] != 0) {
                const int srow = id / KCH;
                if (srow < WROWS) atomicAdd(&corr_row[srow % BM], cweight[s] * cnt[s]);
                else if (!POOL) atomicAdd(&corr_col[(srow - WROWS) % BN], cweight[s] * cnt[s]);
            }
        }
        if constexpr (POOL) {
#pragma unroll
            for (int t = 0; t < PPT; ++t)
                if (tid + t * NT < PITEMS && pl_cnt[t] != 0) atomicAdd(&corr_col[(tid + t * NT) / KT], pl_cnt[t]);
        }
    }
    __syncthreads();  // also: all LDS tile reads are finished, the tile space may be reused

    // ---- weight the plane pairs (Alg. 2) ----
    int val[TM][TN];
#pragma unroll
    for (int r = 0; r < TM; ++r)
#pragma unroll
        for (int c = 0; c < TN; ++c) {
            int v;
            if constexpr (PER_PAIR) {
                v = 0;
#pragma unroll
                for (int i = 0; i < WB; ++i)
#pragma unroll
                    for (int j = 0; j < AB; ++j) v = wrap_add(v, wrap_mul(p.coef[i * 4 + j], acc[i * AB + j][r][c]));
            } else {
                v = acc[0][r][c];
            }
            val[r][c] = v;
        }

    // ---- depth split: the KS wavefronts of an output block add their parts in LDS ----
    if constexpr (KS > 1) {
        int *ctile = reinterpret_cast<int *>(lds);  // [BM][BN]
        if (ks == 0) {
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int c = 0; c < TN; ++c) ctile[(wrow0 + r) * BN + acol0 + c] = val[r][c];
        }
        __syncthreads();
        if (ks != 0) {
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int c = 0; c < TN; ++c) atomicAdd(&ctile[(wrow0 + r) * BN + acol0 + c], val[r][c]);
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < TM; ++r)
#pragma unroll
            for (int c = 0; c < TN; ++c) val[r][c] = ctile[(wrow0 + r) * BN + acol0 + c];
    }
    const bool writer = (ks == 0);

    if (CORR) {
#pragma unroll
        for (int r = 0; r < TM; ++r)
#pragma unroll
            for (int c = 0; c < TN; ++c) val[r][c] = wrap_add(val[r][c], wrap_add(wrap_add(corr_row[wrow0 + r], corr_col[acol0 + c]), p.c0));
    }
    if (XOR) {
#pragma unroll
        for (int r = 0; r < TM; ++r)
#pragma unroll
            for (int c = 0; c < TN; ++c) val[r][c] = wrap_add(val[r][c], p.c0);
    }

    if constexpr (!FUSE) {
        const bool vec_ok = (TN % 4 == 0) && ((p.ldc & 3) == 0) && ((reinterpret_cast<uintptr_t>(p.C) & 15) == 0);
        if (writer) {
#pragma unroll
            for (int r = 0; r < TM; ++r) {
                const int m = m0 + wrow0 + r;
                if (m >= p.M) continue;
                int32_t *crow = p.C + (long long)m * p.ldc;
                const int n = n0 + acol0;
                if (vec_ok && n + TN <= p.N) {
#pragma unroll
                    for (int c = 0; c < TN; c += 4)
                        *reinterpret_cast<int4 *>(crow + n + c) =
                            make_int4(val[r][c], val[r][c + 1], val[r][c + 2], val[r][c + 3]);
                } else {
#pragma unroll
                    for (int c = 0; c < TN; ++c)
                        if (n + c < p.N) crow[n + c] = val[r][c];
                }
            }
        }
    } else {
        // Successive thresholding: count the thresholds reached.  The eight lanes that share a
        // column index hold four consecutive rows each, 32 rows in all: every lane places its
        // results' bits at its rows' positions of one word per plane, three lane exchanges OR the
        // eight partial words together, and the first of the eight lanes stores them (no staging
        // through LDS, no barrier: on the tiny layers that took a quarter of the kernel).
        static_assert(BM % 32 == 0 && TM == 4, "a wavefront's eight row groups of four rows make one 32-bit word");
        if (writer) {  // uniform per wavefront
            uint32_t word[TN][4];
#pragma unroll
            for (int c = 0; c < TN; ++c)
#pragma unroll
                for (int pl = 0; pl < 4; ++pl) word[c][pl] = 0;
            // the threshold count known at compile time, so that a row's thresholds are read from LDS in one
            // go instead of one wait per threshold (rows past M hold INT_MAX thresholds: count 0)
            auto count_rows = [&](auto t_c) {
                constexpr int T = decltype(t_c)::value;
#pragma unroll
                for (int r = 0; r < TM; ++r) {
                    const int *th = thr_s + (wrow0 + r) * T;
                    int tv[T];
#pragma unroll
                    for (int t = 0; t < T; ++t) tv[t] = th[t];
#pragma unroll
                    for (int c = 0; c < TN; ++c) {
                        uint32_t y = 0;
#pragma unroll
                        for (int t = 0; t < T; ++t) y += (val[r][c] >= tv[t]) ? 1u : 0u;
                        // (a row past M holds whatever the unconditional loads brought: its thresholds are INT_MAX, which no
                        // sum within the overflow bound reaches)
#pragma unroll
                        for (int pl = 0; pl < 4; ++pl) word[c][pl] |= ((y >> pl) & 1u) << (4 * ly + r);
                    }
                }
            };
            switch (p.obits) {  // uniform
            case 1: count_rows(std::integral_constant<int, 1>{}); break;
            case 2: count_rows(std::integral_constant<int, 3>{}); break;
            case 3: count_rows(std::integral_constant<int, 7>{}); break;
            default: count_rows(std::integral_constant<int, 15>{}); break;
            }
            const bool last_m_block = (tile_m == p.gy - 1);
            const int wi = m0 / 32 + wm;  // this wavefront's word of the output column
#pragma unroll
            for (int c = 0; c < TN; ++c) {
                const int n = n0 + acol0 + c;
#pragma unroll
                for (int pl = 0; pl < 4; ++pl) {
                    if (pl >= p.obits) break;  // uniform
                    uint32_t v = word[c][pl];
                    v |= __shfl_xor(v, 8);
                    v |= __shfl_xor(v, 16);
                    v |= __shfl_xor(v, 32);
                    if (ly == 0 && n < p.N) {
                        uint32_t *dst = p.Y + ((long long)pl * p.N + n) * p.Yd;
                        dst[wi] = v;
                        // the last row block also clears the padding words of the column
                        if (last_m_block && wm == WM - 1)
                            for (int z = wi + 1; z < p.Yd; ++z) dst[z] = 0;
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------- launch helpers (host)

// Chooses how the tile grid is laid over the 8 XCDs: each gets a compact hy x hx
// rectangle (ry x rx rectangles in all) when the grid is large enough for that to waste
// few workgroups; otherwise plain row-major order.  Returns the number of workgroups.
inline long long plan_tile_order(GemmParams &g, int BM, int BN, int wbits, int abits)
{
    g.gx = (g.N + BN - 1) / BN;
    g.gy = (g.M + BM - 1) / BM;
    g.rx = g.ry = g.hx = g.hy = 0;
    const long long total = (long long)g.gx * g.gy;
    long long best_cost = -1, best_blocks = total;
    const int opts[4][2] = {{4, 2}, {2, 4}, {8, 1}, {1, 8}};  // {ry, rx}
    for (const auto &o : opts) {
        const int ry = o[0], rx = o[1];
        if (g.gy < 2 * ry || g.gx < 2 * rx) continue;
        const int hy = (g.gy + ry - 1) / ry, hx = (g.gx + rx - 1) / rx;
        const long long blocks = 8LL * hy * hx;
        if (blocks * 8 > total * 9) continue;                 // more than 12.5 % surplus workgroups
        // bytes fetched per XCD ~ its weight panel + its activation panel.  Tiles are walked row by row inside
        // a rectangle, so the activation panel is what has to stay in the XCD's L2 from one tile row to the
        // next: among equal fetch costs the narrower rectangle wins (4096^3 W2A2: 36 -> 25 MiB fetched per launch).
        const long long panel = (long long)abits * BN * hx;
        const long long cost = ((long long)wbits * BM * hy + panel) * 4096 + panel / 64;
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost; best_blocks = blocks;
            g.ry = ry; g.rx = rx; g.hy = hy; g.hx = hx;
        }
    }
    return best_blocks;
}

template <int WB, int AB, int TM, int TN, int WM, int WN, int KS, int KT, bool IDLE>
bs_status launch_variant(const GemmParams &g, dim3 grid, bool fuse, bool corr, bool conv, bool xr, hipStream_t st)
{
    dim3 block(WM * WN * KS * 64);
    // A bipolar operand has exactly one plane, so the correction variant only exists
    // where WB == 1 or AB == 1.
    constexpr bool CAN_CORR = (WB == 1 || AB == 1);
    if (corr && !CAN_CORR) return BS_ERR_INVALID_ARG;
    if (xr) {  // both operands bipolar: one plane each
        if constexpr (WB == 1 && AB == 1) {
            if (conv) return BS_ERR_UNSUPPORTED;
            if (fuse) bs_gemm_kernel<1, 1, TM, TN, WM, WN, KS, KT, true, false, false, true, IDLE><<<grid, block, 0, st>>>(g);
            else bs_gemm_kernel<1, 1, TM, TN, WM, WN, KS, KT, false, false, false, true, IDLE><<<grid, block, 0, st>>>(g);
            return bs::after_launch();
        } else {
            return BS_ERR_INVALID_ARG;
        }
    }
    if (conv) {  // implicit lowering exists with the thresholding epilogue only
        if (!fuse) return BS_ERR_UNSUPPORTED;
        if (g.pK > 0) {  // pooled fetch: instantiated for the narrow tiles only (launch_planes takes no other for it)
            if constexpr (KS >= 4 && TN <= 2) {
                if (corr) bs_gemm_kernel<WB, AB, TM, TN, WM, WN, KS, KT, true, CAN_CORR, true, false, IDLE, true><<<grid, block, 0, st>>>(g);
                else bs_gemm_kernel<WB, AB, TM, TN, WM, WN, KS, KT, true, false, true, false, IDLE, true><<<grid, block, 0, st>>>(g);
                return bs::after_launch();
            } else {
                return BS_ERR_UNSUPPORTED;
            }
        }
        if (corr) bs_gemm_kernel<WB, AB, TM, TN, WM, WN, KS, KT, true, CAN_CORR, true, false, IDLE><<<grid, block, 0, st>>>(g);
        else bs_gemm_kernel<WB, AB, TM, TN, WM, WN, KS, KT, true, false, true, false, IDLE><<<grid, block, 0, st>>>(g);
    } else if (fuse) {
        if (corr) bs_gemm_kernel<WB, AB, TM, TN, WM, WN, KS, KT, true, CAN_CORR, false, false, IDLE><<<grid, block, 0, st>>>(g);
        else bs_gemm_kernel<WB, AB, TM, TN, WM, WN, KS, KT, true, false, false, false, IDLE><<<grid, block, 0, st>>>(g);
    } else {
        if (corr) bs_gemm_kernel<WB, AB, TM, TN, WM, WN, KS, KT, false, CAN_CORR, false, false, IDLE><<<grid, block, 0, st>>>(g);
        else bs_gemm_kernel<WB, AB, TM, TN, WM, WN, KS, KT, false, false, false, false, IDLE><<<grid, block, 0, st>>>(g);
    }
    return bs::after_launch();
}

template <int WB, int AB, int TM, int TN, int WM, int WN, int KS, int KT>
bs_status launch_cfg(const GemmParams &g_in, bool fuse, bool corr, bool conv, bool xr, hipStream_t st)
{
    constexpr int BM = 8 * TM * WM, BN = 8 * TN * WN;
    GemmParams g = g_in;
    const long long blocks = plan_tile_order(g, BM, BN, WB, AB);
    if (blocks >= (1LL << 31)) return BS_ERR_UNSUPPORTED;
    finish_params(g);
    dim3 grid((unsigned)blocks);
    // The inner loop's idle-slot rhythm pays when at least two wavefronts share a SIMD.  The small-grid
    // configuration (one wavefront per SIMD and workgroup) gets there only with more workgroups than
    // the chip has compute units.
    if constexpr (KS > 1 && TN == 1) {
        // narrow tiles: the rhythm pays from two workgroups per compute unit on (measured at 516..1024 workgroups:
        // 0..4 % for W1A2, 4..7 % for W2A2 and W4A4)
        if (blocks >= 2 * kIdleMinBlocks) return launch_variant<WB, AB, TM, TN, WM, WN, KS, KT, true>(g, grid, fuse, corr, conv, xr, st);
        return launch_variant<WB, AB, TM, TN, WM, WN, KS, KT, false>(g, grid, fuse, corr, conv, xr, st);
    } else if constexpr (KS > 1 && TN == 4) {
        if (blocks < kIdleMinBlocks) return launch_variant<WB, AB, TM, TN, WM, WN, KS, KT, false>(g, grid, fuse, corr, conv, xr, st);
    }
    return launch_variant<WB, AB, TM, TN, WM, WN, KS, KT, true>(g, grid, fuse, corr, conv, xr, st);
}

template <int WB, int AB>
bs_status launch_planes(const GemmParams &g, bool fuse, bool corr, bool conv, bool xr, hipStream_t st)
{
    // Large grids: 64 x 64 tiles, four wavefronts side by side.  Small grids: 32 x 32
    // tiles whose four wavefronts split the depth, so that more wavefronts exist.  Tiny
    // grids (AlexNet's conv3..conv5 at batch 1: 72 tiles of 32 x 32 on 256 compute units):
    // 32 rows x 8 columns, four times as many workgroups, each with a quarter of the products.
    const long long tiles64 = (long long)((g.M + 63) / 64) * ((g.N + 63) / 64);
    const long long tiles32 = (long long)((g.M + 31) / 32) * ((g.N + 31) / 32);
    constexpr int KT_SMALL = kStageDwords;
    // With more than four plane pairs (the pair-at-a-time loop) a stage of twice the depth halves the barriers per
    // product: 3..13 % on deep products, neutral on short ones (W4A4 256 x 4096 x 256: 22.8 -> 20.2 us; 32 x 32 tiles,
    // 8192 x 8192 x 64: 137 -> 122 us), except where the larger LDS tile limits the resident workgroups (narrow tiles
    // from about 800 workgroups on: 16384 x 4096 x 16 took 45.8 instead of 39.4 us).  One or two pairs measured
    // 5..12 % slower with it, four the same.
    constexpr int KT_DEEP = (WB * AB > 4) ? 2 * kStageDwords : kStageDwords;
    // narrow tiles also whenever at most 16 columns exist: wider tiles would be half empty or more
    if (tiles32 <= kNarrowMaxTiles32 || g.N <= 16) {
        const long long narrow_blocks = (long long)((g.M + 31) / 32) * ((g.N + 7) / 8);
        if (narrow_blocks <= 768) {
            // Eight wavefronts that split stages of twice the depth, instead of four: half as many stages, each with
            // the same products per wavefront, and two wavefronts per SIMD to overlap each other's latencies.  Measured
            // against four (W1A2, W2A2, W4A4; 8..704 workgroups; depth 1024..9216): 6 to 20 % faster for more than four
            // plane pairs at every size, and for up to four pairs from about three stages of depth on while the
            // workgroups do not outnumber the compute units by much (conv4, conv5 of Table 2 at batch 1: 6.8 -> 6.3 and
            // 6.0 -> 5.3 us); up to 38 % slower on short depths with 600 and more workgroups, hence the conditions.
            const bool eight = (WB * AB > 4) || (narrow_blocks <= 400 && g.Kd > 75);
            if (eight) return launch_cfg<WB, AB, 4, 1, 1, 1, 8, 2 * kStageDwords>(g, fuse, corr, conv, xr, st);
            return launch_cfg<WB, AB, 4, 1, 1, 1, 4, KT_DEEP>(g, fuse, corr, conv, xr, st);
        }
        return launch_cfg<WB, AB, 4, 1, 1, 1, 4, KT_SMALL>(g, fuse, corr, conv, xr, st);
    }
    // just above the tiny grids 32 x 16 tiles still pay: twice the workgroups, so that two wavefronts share a SIMD
    // (4096 x 9216 x 64 W1A2: 18.7 -> 15.5 us; W4A4 4096 x 4096 x 64: 49.9 -> 41.5 us; a tie from 512 tiles on)
    // (also for every larger grid with a pooled fetch, whose kernels exist for the narrow tiles only: a thread of
    // a wider tile would have to hold the window taps of eight and more words per stage)
    if (tiles32 <= kHalfWidthMaxTiles32 || (conv && g.pK > 0)) return launch_cfg<WB, AB, 4, 2, 1, 1, 4, KT_DEEP>(g, fuse, corr, conv, xr, st);
    if (tiles64 < kWideMinTiles64) return launch_cfg<WB, AB, 4, 4, 1, 1, 4, KT_DEEP>(g, fuse, corr, conv, xr, st);
    return launch_cfg<WB, AB, 4, 4, 2, 2, 1, kStageDwords>(g, fuse, corr, conv, xr, st);
}

// Defined once per WB in bs_gemm_w<WB>.hip (explicit instantiation) to keep builds parallel.
template <int WB>
bs_status launch_wb(const GemmParams &g, int abits, bool fuse, bool corr, bool conv, bool xr, hipStream_t st)
{
    switch (abits) {
    case 1: return launch_planes<WB, 1>(g, fuse, corr, conv, xr, st);
    case 2: return launch_planes<WB, 2>(g, fuse, corr, conv, xr, st);
    case 3: return launch_planes<WB, 3>(g, fuse, corr, conv, xr, st);
    default: return launch_planes<WB, 4>(g, fuse, corr, conv, xr, st);
    }
}

}  // namespace bs
