// Bit-serial GEMV: the bit-serial GEMM of Alg. 2 for a handful of columns (batch-1
// fully-connected layers, Table 2's (4096, 9216, 1) and (4096, 4096, 1)).  Every weight
// bit is read exactly once and used for N <= 4 columns, so the kernel is a stream over
// the packed weight planes bound by HBM, not by popcount throughput.
//
// Shape: one wavefront per workgroup, eight rows per wavefront, eight lanes per row.
// The eight lanes of a row read consecutive 16-byte chunks (one full 128-byte line per
// load and row) and stride over the depth; the activation planes sit in LDS, read with
// broadcast.  Several loads per lane are issued before the first use so that enough
// bytes are in flight.  The eight partial sums of a row are combined with lane
// exchanges; the row leaders apply the plane-pair weights (Alg. 2), the bipolar
// correction and, if asked, successive thresholding, and a ballot turns the eight
// results into one output byte per plane and column.
#include "bs_gemm_kernel.h"

namespace bs {
namespace {

constexpr int ROWS_PER_WAVE = 8;   // also the bits of one output byte
constexpr int LANES_PER_ROW = 8;
constexpr int UNROLL = 4;          // chunks per lane and plane in flight

template <int WB, int AB, int NC, bool FUSE>
__global__ void __launch_bounds__(64) bs_gemv_kernel(const GemmParams p)
{
    extern __shared__ uint4 ldsA[];  // [AB][NC][nch]
    const int lane = threadIdx.x;
    const int nch = p.Kd >> 2;       // 16-byte chunks per packed row

    // ---- activation planes -> LDS, and their weighted popcounts (bipolar weights) ----
    int colsum[NC];
#pragma unroll
    for (int n = 0; n < NC; ++n) colsum[n] = 0;
    {
        const uint4 *Ag = reinterpret_cast<const uint4 *>(p.A);
        const int total = AB * NC * nch;
        for (int id = lane; id < total; id += 64) {
            const int c = id % nch, jn = id / nch;
            const int n = jn % NC, j = jn / NC;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (n < p.N) v = Ag[(size_t)(j * p.N + n) * nch + c];
            ldsA[id] = v;
            const int pc = popc4(v) * p.ccol[j];
#pragma unroll
            for (int nn = 0; nn < NC; ++nn) colsum[nn] += (nn == n) ? pc : 0;
        }
#pragma unroll
        for (int n = 0; n < NC; ++n)
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) colsum[n] += __shfl_xor(colsum[n], o);
    }
    __syncthreads();

    const int g = lane & (LANES_PER_ROW - 1), r = lane / LANES_PER_ROW;
    const int m = blockIdx.x * ROWS_PER_WAVE + r;
    const bool mvalid = m < p.M;
    const uint4 *Wg = reinterpret_cast<const uint4 *>(p.W);

    int acc[WB * AB][NC];
#pragma unroll
    for (int q = 0; q < WB * AB; ++q)
#pragma unroll
        for (int n = 0; n < NC; ++n) acc[q][n] = 0;

    for (int c0 = g; c0 < nch; c0 += LANES_PER_ROW * UNROLL) {
        uint4 w[UNROLL][WB];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = c0 + u * LANES_PER_ROW;
#pragma unroll
            for (int i = 0; i < WB; ++i) {
                w[u][i] = make_uint4(0, 0, 0, 0);
                if (mvalid && c < nch) w[u][i] = Wg[(size_t)(i * p.M + m) * nch + c];
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = c0 + u * LANES_PER_ROW;
            if (c < nch) {
#pragma unroll
                for (int j = 0; j < AB; ++j)
#pragma unroll
                    for (int n = 0; n < NC; ++n) {
                        const uint4 a = ldsA[(j * NC + n) * nch + c];
#pragma unroll
                        for (int i = 0; i < WB; ++i) acc[i * AB + j][n] = popc_and4(w[u][i], a, acc[i * AB + j][n]);
                    }
            }
        }
    }

    // ---- plane-pair weighting (Alg. 2), reduction over the lanes of a row ----
    int val[NC];
#pragma unroll
    for (int n = 0; n < NC; ++n) {
        int v = 0;
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
            for (int j = 0; j < AB; ++j) v += p.coef[i * 4 + j] * acc[i * AB + j][n];
#pragma unroll
        for (int o = LANES_PER_ROW / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
        val[n] = v + colsum[n];
    }
    const bool leader = (g == 0) && mvalid;

    if constexpr (!FUSE) {
        if (leader) {
#pragma unroll
            for (int n = 0; n < NC; ++n)
                if (n < p.N) p.C[(long long)m * p.ldc + n] = val[n];
        }
    } else {
        uint8_t *Yb = reinterpret_cast<uint8_t *>(p.Y);
        const long long col_bytes = (long long)p.Yd * 4;
        int y[NC];
#pragma unroll
        for (int n = 0; n < NC; ++n) y[n] = 0;
        if (leader) {
            const int32_t *th = p.thr + (long long)m * p.T;
            for (int t = 0; t < p.T; ++t) {
                const int32_t tv = th[t];
#pragma unroll
                for (int n = 0; n < NC; ++n) y[n] += (val[n] >= tv) ? 1 : 0;
            }
        }
        for (int pl = 0; pl < p.obits; ++pl) {
#pragma unroll
            for (int n = 0; n < NC; ++n) {
                if (n < p.N) {
                    // leaders sit at lanes 0, 8, ..., 56: gather those eight bits into a byte
                    const unsigned long long mask = __ballot(leader && ((y[n] >> pl) & 1));
                    const unsigned byte = (unsigned)((mask * 0x0102040810204080ull) >> 56);
                    if (lane == 0) Yb[((long long)pl * p.N + n) * col_bytes + blockIdx.x] = (uint8_t)byte;
                }
            }
        }
        // the last workgroup clears the padding bytes of every column
        if (blockIdx.x == gridDim.x - 1) {
            const int first = gridDim.x, npad = (int)col_bytes - first;
            for (int it = lane; it < npad * p.obits * p.N; it += 64) {
                const int z = it % npad, cn = it / npad;
                Yb[(long long)cn * col_bytes + first + z] = 0;
            }
        }
    }
}

template <int WB, int AB, int NC>
bs_status launch_gemv_nc(const GemmParams &g, bool fuse, size_t lds_bytes, hipStream_t st)
{
    dim3 grid((unsigned)((g.M + ROWS_PER_WAVE - 1) / ROWS_PER_WAVE));
    if (fuse) bs_gemv_kernel<WB, AB, NC, true><<<grid, 64, lds_bytes, st>>>(g);
    else bs_gemv_kernel<WB, AB, NC, false><<<grid, 64, lds_bytes, st>>>(g);
    return after_launch();
}

template <int WB, int AB>
bs_status launch_gemv_ab(const GemmParams &g, bool fuse, hipStream_t st)
{
    const int nc = g.N == 1 ? 1 : (g.N == 2 ? 2 : 4);
    const size_t lds_bytes = (size_t)AB * nc * (g.Kd >> 2) * 16;
    switch (nc) {
    case 1: return launch_gemv_nc<WB, AB, 1>(g, fuse, lds_bytes, st);
    case 2: return launch_gemv_nc<WB, AB, 2>(g, fuse, lds_bytes, st);
    default: return launch_gemv_nc<WB, AB, 4>(g, fuse, lds_bytes, st);
    }
}

template <int WB>
bs_status launch_gemv_wb(const GemmParams &g, int abits, bool fuse, hipStream_t st)
{
    switch (abits) {
    case 1: return launch_gemv_ab<WB, 1>(g, fuse, st);
    case 2: return launch_gemv_ab<WB, 2>(g, fuse, st);
    case 3: return launch_gemv_ab<WB, 3>(g, fuse, st);
    default: return launch_gemv_ab<WB, 4>(g, fuse, st);
    }
}

}  // namespace

bool gemv_applicable(const GemmParams &g, int abits, bool a_bipolar)
{
    if (g.N > kGemvMaxCols || a_bipolar) return false;
    const int nc = g.N == 1 ? 1 : (g.N == 2 ? 2 : 4);
    return (size_t)abits * nc * (g.Kd >> 2) * 16 <= kGemvMaxLds;
}

bs_status launch_gemv(const GemmParams &g, int wbits, int abits, bool fuse, hipStream_t st)
{
    switch (wbits) {
    case 1: return launch_gemv_wb<1>(g, abits, fuse, st);
    case 2: return launch_gemv_wb<2>(g, abits, fuse, st);
    case 3: return launch_gemv_wb<3>(g, abits, fuse, st);
    default: return launch_gemv_wb<4>(g, abits, fuse, st);
    }
}

}  // namespace bs
