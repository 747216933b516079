#pragma once
// Bit-serial GEMV: the bit-serial GEMM of Alg. 2 for a handful of columns (batch-1
// fully-connected layers, Table 2's (4096, 9216, 1) and (4096, 4096, 1)).  A workgroup
// reads every weight bit of its rows exactly once and uses it for up to four columns, so
// the kernel is a stream over the packed weight planes bound by HBM, not by popcount
// throughput.  Five to sixteen columns run as groups of four in the grid's second
// dimension; the groups run side by side and find the weights of the others in L2.
//
// Shape: a workgroup of four wavefronts owns eight rows (one output byte per plane and
// column); 32 lanes share a row and read consecutive 16-byte chunks, so one load
// instruction of a wavefront covers two 512-byte runs.  The weight stream is started
// before anything else; the (small) activation planes are then copied to LDS, where all
// rows read them with broadcast.  The 32 partial sums of a row are combined with lane
// exchanges; the row leaders apply the plane-pair weights (Alg. 2), the bipolar
// correction and, if asked, successive thresholding; the eight results of the workgroup
// meet in LDS and leave as one byte per plane and column.
#include "bs_gemm_kernel.h"

namespace bs {

constexpr int ROWS_PER_BLOCK = 8;   // also the bits of one output byte
constexpr int LANES_PER_ROW = 32;
constexpr int GEMV_THREADS = ROWS_PER_BLOCK * LANES_PER_ROW;

// Pooled activation fill: item id = n * (Kd / VW) + u is unit u (VW = 1 or 4 words) of column n, i.e. words
// q = u * VW .. of the flattened pooled map of image n0 + n; issue() requests the window taps of all planes, store()
// takes their bit-sliced maximum, writes it to the planes in LDS ([AB][NC][Kd] words) and counts its bits.
template <int AB, int NC, typename V>
struct PoolFill {
    static constexpr int VW = sizeof(V) / 4;
    V raw[9][AB];
    uint32_t keep;
    __device__ __forceinline__ void locate(const GemmParams &p, int id, int &n, int &q) const
    {
        const int units = p.Kd / VW;
        n = 0;
#pragma unroll
        for (int z = 0; z < NC; ++z)
            if (id >= units) { id -= units; ++n; }
        q = id * VW;
    }
    __device__ __forceinline__ void issue(const GemmParams &p, int id, int n0)
    {
        int n, q;
        locate(p, id, n, q);
        const bool ok = n < NC && q < p.cKused && n0 + n < p.N;
        const int tap = fdiv(q, p.dCd), cd = q - tap * p.cCd;
        const int fr = fdiv(tap, p.dKW), fs = tap - fr * p.cKW;  // pixel of the pooled map
        const int at = ((n0 + n) * p.pH * p.pW + fr * p.pS * p.pW + fs * p.pS) * p.cPix + cd;
        pool_load<AB, V>(p.A, p.cB * p.pH * p.pW * p.cPix, at, p.pW * p.cPix, p.cPix, p.pK, ok, raw);
        keep = ok ? 0xFFFFFFFFu : 0u;
    }
    __device__ __forceinline__ void store(const GemmParams &p, int id, uint32_t *lds_words, int (&colsum)[NC]) const
    {
        int n, q;
        locate(p, id, n, q);
        if (n >= NC) return;
        V best[AB];
        pool_max<AB, V>(raw, keep, best);
#pragma unroll
        for (int j = 0; j < AB; ++j) {
            *reinterpret_cast<V *>(lds_words + (j * NC + n) * p.Kd + q) = best[j];
            int pc;
            if constexpr (VW == 1) pc = __popc(best[j]);
            else if constexpr (VW == 2) pc = __popc(best[j].x) + __popc(best[j].y);
            else pc = __popc(best[j].x) + __popc(best[j].y) + __popc(best[j].z) + __popc(best[j].w);
            pc *= p.ccol[j];
#pragma unroll
            for (int nn = 0; nn < NC; ++nn) colsum[nn] += (nn == n) ? pc : 0;
        }
    }
};

// NT: read the weights with the non-temporal hint (large weight sets, single column).
// POOL: a column is not a packed row in memory but the flattened maximum over pK x pK windows of image n of an
// unpooled map (a fully connected layer behind a pooling layer, i.e. a convolution whose kernel covers the whole
// pooled map): the fill of the activation planes forms each 32-channel word from its window, all planes at once.
// UNROLL: chunks per lane and plane fetched in one go (1..4): the groups of 32 chunks a row holds, so that no load of
// the burst is redundant (W4A4, depth 8192: two groups; with four, half of the loads re-read the last chunk and the
// kernel took 12.9 instead of 9.5 us).
template <int WB, int AB, int NC, int UNROLL, bool FUSE, bool XOR = false, bool NT = false, bool POOL = false>
__global__ void __launch_bounds__(GEMV_THREADS) bs_gemv_kernel(const GemmParams p)
{
    bs::prefetch_kernel_arguments<(int)sizeof(GemmParams)>();
    extern __shared__ uint4 ldsA[];  // [AB][NC][nch]
    __shared__ int colsum_s[NC];
    __shared__ int yrow[ROWS_PER_BLOCK][NC];
    const int tid = threadIdx.x;
    const int nch = p.Kd >> 2;       // 16-byte chunks per packed row

    const int g = tid & (LANES_PER_ROW - 1), r = tid / LANES_PER_ROW;
    const int m = blockIdx.x * ROWS_PER_BLOCK + r;
    const int n0 = blockIdx.y * NC;  // first column of this workgroup's group (more than NC columns: several groups)
    const bool mvalid = m < p.M;
    const uint4 *Wg = reinterpret_cast<const uint4 *>(p.W);

    uint4 w[UNROLL][WB];
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    // Unconditional loads: a row past M reads the last row (its results are never stored) and a chunk past the depth
    // the last chunk (its products are skipped).  Behind a load that sits in a branch the compiler cannot count how
    // many loads follow an earlier one and waits for all of them (s_waitcnt vmcnt(0)); with a straight-line burst
    // it waits chunk by chunk, so a lane multiplies its first chunks while the later ones are still arriving.
    const int m_safe = mvalid ? m : p.M - 1;
    auto fetch_w = [&](int c0) {
        // Weight sets too large to stay in the last-level cache are read with the
        // non-temporal hint (measured on a 134 MB stream: 4.4 -> 5.1 TB/s); smaller ones
        // are left cacheable so that repeated inference finds them on chip.
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = c0 + u * LANES_PER_ROW, c_safe = c < nch ? c : nch - 1;
#pragma unroll
            for (int i = 0; i < WB; ++i) {
                const uint4 *src = Wg + (size_t)(i * p.M + m_safe) * nch + c_safe;
                if constexpr (NT) {
                    const v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(src));
                    w[u][i] = make_uint4(t.x, t.y, t.z, t.w);
                } else {
                    w[u][i] = *src;
                }
            }
        }
    };
    // POOL: the activation fill forms pooled words instead of copying.  The first items' window loads are requested even
    // before the weights: they return first, and the comparisons run while the weight stream is on its way.
    // One 32-channel word per item, two items per thread and trip.  (Wider items, i.e. fewer and wider loads, measured
    // slower: fc6 behind pool5 takes 5.1 us with one word per item, 5.7 with two, 6.2 with four; the comparisons then
    // sit in fewer wavefronts.)
    PoolFill<AB, NC, uint32_t> fill[2];
    if constexpr (POOL) {
#pragma unroll
        for (int h = 0; h < 2; ++h) fill[h].issue(p, tid + h * GEMV_THREADS, n0);
    }
    // Row leaders fetch their thresholds first of all, so that the epilogue does not wait for a second round trip to
    // memory (these loads sit in branches and must not follow the weight burst, see fetch_w).
    int32_t thv[FUSE ? 15 : 1];
    if constexpr (FUSE) {
#pragma unroll
        for (int t = 0; t < 15; ++t) {
            thv[t] = 0x7fffffff;
            if (g == 0 && mvalid && t < p.T) thv[t] = p.thr[(long long)m * p.T + t];
        }
    }
    // The first two trips of the activation fill are requested before the weights.  Loads return in order: behind the
    // weight burst its words would arrive last, and the fill, the barrier behind it and with them all arithmetic
    // would wait for the whole burst; ahead of it they arrive first and the products of a lane's first chunks run while
    // its later chunks are still on their way.
    const uint4 *Ag = reinterpret_cast<const uint4 *>(p.A);
    const int total = POOL ? 0 : AB * NC * nch;
    auto act_chunk = [&](int id) -> uint4 {
        const int c = id % nch, jn = id / nch;
        const int n = jn % NC, j = jn / NC;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (id < total && n0 + n < p.N) v = Ag[(size_t)(j * p.N + n0 + n) * nch + c];
        return v;
    };
    const uint4 act_first[2] = {act_chunk(tid), act_chunk(tid + GEMV_THREADS)};  // two trips cover 8 KB of planes
    fetch_w(g);

    // ---- activation planes -> LDS, and their weighted popcounts (bipolar weights) ----
    if (tid < NC) colsum_s[tid] = 0;
    __syncthreads();
    {
        int colsum[NC];
#pragma unroll
        for (int n = 0; n < NC; ++n) colsum[n] = 0;
        if constexpr (POOL) {
            uint32_t *ldsD = reinterpret_cast<uint32_t *>(ldsA);
            for (int id = tid; id < NC * p.Kd; id += 2 * GEMV_THREADS) {
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    if (id != tid) fill[h].issue(p, id + h * GEMV_THREADS, n0);
#pragma unroll
                for (int h = 0; h < 2; ++h) fill[h].store(p, id + h * GEMV_THREADS, ldsD, colsum);
            }
        }
        for (int id = tid; id < total; id += GEMV_THREADS) {
            const int n = (id / nch) % NC, j = (id / nch) / NC;
            const uint4 v = id == tid ? act_first[0] : (id == tid + GEMV_THREADS ? act_first[1] : act_chunk(id));
            ldsA[id] = v;
            // the plane's weight by selects: indexing the kernel arguments with a per-lane j would be a vector load
            // from memory, which returns behind the whole weight burst and would make the fill wait for it
            int cc = p.ccol[0];
#pragma unroll
            for (int jj = 1; jj < AB; ++jj) cc = (j == jj) ? p.ccol[jj] : cc;
            const int pc = popc4(v) * cc;
#pragma unroll
            for (int nn = 0; nn < NC; ++nn) colsum[nn] += (nn == n) ? pc : 0;
        }
        if (p.ccol[0] != 0) {  // only a bipolar weight operand needs the column term
#pragma unroll
            for (int n = 0; n < NC; ++n) {
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) colsum[n] += __shfl_xor(colsum[n], o);
                if ((tid & 63) == 0) atomicAdd(&colsum_s[n], colsum[n]);
            }
        }
    }
    __syncthreads();

    int acc[WB * AB][NC];
#pragma unroll
    for (int q = 0; q < WB * AB; ++q)
#pragma unroll
        for (int n = 0; n < NC; ++n) acc[q][n] = 0;

    for (int c0 = g; c0 < nch; c0 += LANES_PER_ROW * UNROLL) {
        if (c0 != g) fetch_w(c0);
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
                        for (int i = 0; i < WB; ++i)
                            acc[i * AB + j][n] = XOR ? popc_xor4(w[u][i], a, acc[i * AB + j][n]) : popc_and4(w[u][i], a, acc[i * AB + j][n]);
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
            for (int j = 0; j < AB; ++j) v = wrap_add(v, wrap_mul(p.coef[i * 4 + j], acc[i * AB + j][n]));
#pragma unroll
        for (int o = LANES_PER_ROW / 2; o > 0; o >>= 1) v = wrap_add(v, __shfl_xor(v, o));
        val[n] = wrap_add(v, wrap_add(colsum_s[n], p.c0));
    }
    const bool leader = (g == 0) && mvalid;

    if constexpr (!FUSE) {
        if (leader) {
#pragma unroll
            for (int n = 0; n < NC; ++n)
                if (n0 + n < p.N) p.C[(long long)m * p.ldc + n0 + n] = val[n];
        }
    } else {
        uint8_t *Yb = reinterpret_cast<uint8_t *>(p.Y);
        const long long col_bytes = (long long)p.Yd * 4;
        if (g == 0) {
            int y[NC];
#pragma unroll
            for (int n = 0; n < NC; ++n) y[n] = 0;
            if (mvalid) {
#pragma unroll
                for (int t = 0; t < 15; ++t) {
                    if (t < p.T) {
#pragma unroll
                        for (int n = 0; n < NC; ++n) y[n] += (val[n] >= thv[t]) ? 1 : 0;
                    }
                }
            }
#pragma unroll
            for (int n = 0; n < NC; ++n) yrow[r][n] = y[n];
        }
        __syncthreads();
        // thread (pl, n) assembles the byte of plane pl, column n from the eight rows
        if (tid < p.obits * NC) {
            const int pl = tid / NC, n = tid % NC;
            if (n0 + n < p.N) {
                unsigned byte = 0;
#pragma unroll
                for (int rr = 0; rr < ROWS_PER_BLOCK; ++rr) byte |= ((yrow[rr][n] >> pl) & 1u) << rr;
                Yb[((long long)pl * p.N + n0 + n) * col_bytes + blockIdx.x] = (uint8_t)byte;
            }
        }
        // the last workgroup (of the first column group) clears the padding bytes of every column
        if (blockIdx.x == gridDim.x - 1 && blockIdx.y == 0) {
            const int first = gridDim.x, npad = (int)col_bytes - first;
            for (int it = tid; it < npad * p.obits * p.N; it += GEMV_THREADS) {
                const int z = it % npad, cn = it / npad;
                Yb[(long long)cn * col_bytes + first + z] = 0;
            }
        }
    }
}

// Chunks per lane fetched in one go: all groups of 32 chunks of a row when there are at most four, else the count
// among 4, 3, 2 that leaves the fewest redundant groups in the last trip.
inline int gemv_unroll(int nch)
{
    const int groups = (nch + LANES_PER_ROW - 1) / LANES_PER_ROW;
    if (groups <= 4) return groups;
    int best = 4, waste = (4 - groups % 4) % 4;
    for (int u = 3; u >= 2; --u)
        if ((u - groups % u) % u < waste) { best = u; waste = (u - groups % u) % u; }
    return best;
}

template <int WB, int AB, int NC, int U>
bs_status launch_gemv_u(const GemmParams &g, bool fuse, bool xr, size_t lds_bytes, hipStream_t st)
{
    dim3 grid((unsigned)((g.M + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK), (unsigned)((g.N + NC - 1) / NC));
    if (xr) {
        if constexpr (WB == 1 && AB == 1) {
            if (fuse) bs_gemv_kernel<1, 1, NC, U, true, true><<<grid, GEMV_THREADS, lds_bytes, st>>>(g);
            else bs_gemv_kernel<1, 1, NC, U, false, true><<<grid, GEMV_THREADS, lds_bytes, st>>>(g);
            return after_launch();
        } else {
            return BS_ERR_INVALID_ARG;
        }
    }
    if (g.pK > 0) {  // pooled columns: with the thresholding epilogue only
        if (!fuse) return BS_ERR_UNSUPPORTED;
        bs_gemv_kernel<WB, AB, NC, U, true, false, false, true><<<grid, GEMV_THREADS, lds_bytes, st>>>(g);
        return after_launch();
    }
    if constexpr (NC == 1 && U == 4) {  // weight sets of 64 MB and more have many groups per row: four at a time
        if (g.stream_weights) {
            if (fuse) bs_gemv_kernel<WB, AB, 1, 4, true, false, true><<<grid, GEMV_THREADS, lds_bytes, st>>>(g);
            else bs_gemv_kernel<WB, AB, 1, 4, false, false, true><<<grid, GEMV_THREADS, lds_bytes, st>>>(g);
            return after_launch();
        }
    }
    if (fuse) bs_gemv_kernel<WB, AB, NC, U, true><<<grid, GEMV_THREADS, lds_bytes, st>>>(g);
    else bs_gemv_kernel<WB, AB, NC, U, false><<<grid, GEMV_THREADS, lds_bytes, st>>>(g);
    return after_launch();
}

template <int WB, int AB, int NC>
bs_status launch_gemv_nc(const GemmParams &g, bool fuse, bool xr, size_t lds_bytes, hipStream_t st)
{
    const int u = (NC == 1 && g.stream_weights && g.pK == 0 && !xr) ? 4 : gemv_unroll(g.Kd >> 2);
    switch (u) {
    case 1: return launch_gemv_u<WB, AB, NC, 1>(g, fuse, xr, lds_bytes, st);
    case 2: return launch_gemv_u<WB, AB, NC, 2>(g, fuse, xr, lds_bytes, st);
    case 3: return launch_gemv_u<WB, AB, NC, 3>(g, fuse, xr, lds_bytes, st);
    default: return launch_gemv_u<WB, AB, NC, 4>(g, fuse, xr, lds_bytes, st);
    }
}

template <int WB, int AB>
bs_status launch_gemv_ab(const GemmParams &g, bool fuse, bool xr, hipStream_t st)
{
    const int nc = g.N == 1 ? 1 : (g.N == 2 ? 2 : 4);
    const size_t lds_bytes = (size_t)AB * nc * (g.Kd >> 2) * 16;
    switch (nc) {
    case 1: return launch_gemv_nc<WB, AB, 1>(g, fuse, xr, lds_bytes, st);
    case 2: return launch_gemv_nc<WB, AB, 2>(g, fuse, xr, lds_bytes, st);
    default: return launch_gemv_nc<WB, AB, 4>(g, fuse, xr, lds_bytes, st);
    }
}

template <int WB>
bs_status launch_gemv_wb(const GemmParams &g, int abits, bool fuse, bool xr, hipStream_t st)
{
    switch (abits) {
    case 1: return launch_gemv_ab<WB, 1>(g, fuse, xr, st);
    case 2: return launch_gemv_ab<WB, 2>(g, fuse, xr, st);
    case 3: return launch_gemv_ab<WB, 3>(g, fuse, xr, st);
    default: return launch_gemv_ab<WB, 4>(g, fuse, xr, st);
    }
}


}  // namespace bs
