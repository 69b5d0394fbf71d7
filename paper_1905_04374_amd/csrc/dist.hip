// Distance pass: all pairwise squared l2 distances between the n gradients
// (Algorithm 1, multi-Krum, the score line; Eq. 4), computed once per
// aggregation (Section V-B).
//
// Two evaluations, both streaming every gradient from HBM exactly once and
// both free of atomics, so that results depend on the data only:
//
//  direct: sum_c (x_i[c]-x_j[c])^2 on the vector ALU.  A workgroup of 16 waves
//          stages a tile of n x 128 coordinates in LDS; wave w owns one 8x8
//          block of row pairs and keeps its 64 partial sums in registers
//          (lane = coordinate).  n(n-1) lane-operations per coordinate.
//
//  gram:   G = X X^T on the fp32 matrix cores (v_mfma_f32_16x16x4_f32), the
//          rows padded to blocks of 16 and only the lower block triangle
//          computed; D_ij = G_ii + G_jj - 2 G_ij afterwards in fp64.  The
//          MFMA accumulators are fp32 and are flushed into fp64 running sums
//          every 256 coordinates, which keeps the cancellation in the last
//          formula harmless.  Each lane loads 16 bytes of one row straight
//          into the operand layout of the instruction (row = lane%16,
//          k-slice = lane/16), no LDS staging.
//
// Every workgroup writes its partial sums as doubles; a second kernel adds
// them over workgroups in index order and a third forms the n x n matrix.
#include <hip/hip_runtime.h>

#include "mb_internal.hpp"

namespace mb {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ direct
constexpr int kDirThreads = 1024;  // 16 waves
constexpr int kDirTile = 128;      // coordinates per LDS tile
constexpr int kRB = 8;             // rows per block of the pair blocking

// block pair index bp -> (I, J), I >= J, bp = I(I+1)/2 + J
__device__ __forceinline__ void unpack_pair(int bp, int &I, int &J)
{
    int i = 0;
    while ((i + 1) * (i + 2) / 2 <= bp) ++i;
    I = i;
    J = bp - i * (i + 1) / 2;
}

__global__ __launch_bounds__(kDirThreads) void dist_direct_kernel(
    const float *__restrict__ G, int n, int64_t d, int64_t ld, double *__restrict__ partials,
    int npairs_blocks)
{
    __shared__ float tile[kMaxN][kDirTile];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int bp = blockIdx.y * 16 + wave;      // this wave's block pair
    const bool have_pair = bp < npairs_blocks;
    int I = 0, J = 0;
    if (have_pair) unpack_pair(bp, I, J);
    const int nrows = ((n + kRB - 1) / kRB) * kRB;  // rows staged (padded rows are zero)

    float acc[kRB][kRB];
#pragma unroll
    for (int a = 0; a < kRB; ++a)
#pragma unroll
        for (int b = 0; b < kRB; ++b) acc[a][b] = 0.0f;

    const int64_t ntiles = (d + kDirTile - 1) / kDirTile;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t c0 = t * kDirTile;
        // stage: element e -> row e/128, column e%128 (coalesced along the row)
        for (int e = tid; e < nrows * kDirTile; e += kDirThreads) {
            const int r = e / kDirTile, c = e % kDirTile;
            float x = 0.0f;
            if (r < n && c0 + c < d) x = G[(int64_t)r * ld + c0 + c];
            tile[r][c] = x;
        }
        __syncthreads();
        if (have_pair) {
#pragma unroll
            for (int h = 0; h < kDirTile / 64; ++h) {
                const int c = h * 64 + lane;
                float xi[kRB], xj[kRB];
#pragma unroll
                for (int a = 0; a < kRB; ++a) {
                    xi[a] = tile[I * kRB + a][c];
                    xj[a] = tile[J * kRB + a][c];
                }
#pragma unroll
                for (int a = 0; a < kRB; ++a)
#pragma unroll
                    for (int b = 0; b < kRB; ++b) {
                        const float df = xi[a] - xj[b];
                        acc[a][b] = fmaf(df, df, acc[a][b]);
                    }
            }
        }
        __syncthreads();
    }
    if (!have_pair) return;
    // sum over the 64 lanes in a fixed butterfly order, then one double per pair entry
    double *dst = partials + ((int64_t)blockIdx.x * 36 + bp) * 64;
#pragma unroll
    for (int a = 0; a < kRB; ++a)
#pragma unroll
        for (int b = 0; b < kRB; ++b) {
            double s = (double)acc[a][b];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
            if (lane == 0) dst[a * kRB + b] = s;
        }
}

// reduced[bp*64 + a*8 + b] holds sum_c (x_{8I+a} - x_{8J+b})^2
__global__ void finalize_direct_kernel(const double *__restrict__ reduced, int n,
                                       double *__restrict__ dist, int accumulate)
{
    for (int e = threadIdx.x; e < n * n; e += blockDim.x) {
        const int i = e / n, j = e % n;
        const int hi = i > j ? i : j, lo = i > j ? j : i;
        double v = 0.0;
        if (hi != lo) {
            const int I = hi / kRB, J = lo / kRB;
            const int bp = I * (I + 1) / 2 + J;
            v = reduced[bp * 64 + (hi % kRB) * kRB + (lo % kRB)];
        }
        dist[e] = accumulate ? dist[e] + v : v;
    }
}

// -------------------------------------------------------------------- gram
constexpr int kGramThreads = 256;  // 4 waves, each streaming its own columns
constexpr int kGramCols = 32;      // columns per wave step (two 16-byte loads per lane and row block)
constexpr int kFlush = 8;          // steps between flushes of the fp32 accumulators into fp64

template <int NB>
struct GramAcc {
    static constexpr int NT = NB * (NB + 1) / 2;
    floatx4 acc[NT];
    double sum[NT][4];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int v = 0; v < 4; ++v) sum[t][v] = 0.0;
        }
    }
    __device__ __forceinline__ void flush()
    {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int v = 0; v < 4; ++v) sum[t][v] += (double)acc[t][v];
            acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    }
    // one k-slice: x[I] = this lane's value of row block I
    __device__ __forceinline__ void mac(const float (&x)[NB])
    {
        int t = 0;
#pragma unroll
        for (int I = 0; I < NB; ++I)
#pragma unroll
            for (int J = 0; J <= I; ++J, ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[I], x[J], acc[t], 0, 0, 0);
    }
};

template <int NB, bool ALIGNED>
__global__ __launch_bounds__(kGramThreads) void dist_gram_kernel(
    const float *__restrict__ G, int n, int64_t d, int64_t ld, double *__restrict__ partials)
{
    constexpr int NT = NB * (NB + 1) / 2;
    __shared__ double red[NT * 256];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15;   // row within a block of 16
    const int q = lane >> 4;   // k-slice
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t gw = (int64_t)blockIdx.x * 4 + wave;

    const float *rowp[NB];
    bool rowok[NB];
#pragma unroll
    for (int I = 0; I < NB; ++I) {
        const int row = 16 * I + r;
        rowok[I] = row < n;
        rowp[I] = G + (int64_t)(rowok[I] ? row : 0) * ld;
    }

    GramAcc<NB> g;
    g.clear();
    const int64_t nfull = ALIGNED ? d / kGramCols : 0;   // steps made of whole 16-byte loads
    int since_flush = 0;

    if constexpr (ALIGNED) {
        float4 a0[NB], a1[NB];
        int64_t t = gw;
        auto load = [&](int64_t step) {
            const int64_t c = step * kGramCols + 4 * q;
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                if (rowok[I]) {
                    a0[I] = *reinterpret_cast<const float4 *>(rowp[I] + c);
                    a1[I] = *reinterpret_cast<const float4 *>(rowp[I] + c + 16);
                } else {
                    a0[I] = make_float4(0.f, 0.f, 0.f, 0.f);
                    a1[I] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        };
        if (t < nfull) load(t);
        while (t < nfull) {
            float4 b0[NB], b1[NB];
#pragma unroll
            for (int I = 0; I < NB; ++I) { b0[I] = a0[I]; b1[I] = a1[I]; }
            const int64_t tn = t + nwaves;
            if (tn < nfull) load(tn);     // next step's loads fly while this step multiplies
            float x[NB];
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = b0[I].x;
            g.mac(x);
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = b0[I].y;
            g.mac(x);
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = b0[I].z;
            g.mac(x);
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = b0[I].w;
            g.mac(x);
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = b1[I].x;
            g.mac(x);
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = b1[I].y;
            g.mac(x);
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = b1[I].z;
            g.mac(x);
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = b1[I].w;
            g.mac(x);
            if (++since_flush == kFlush) { g.flush(); since_flush = 0; }
            t = tn;
        }
    }
    // remaining columns (all of them on the unaligned path), 4 per step and lane group,
    // element-wise guarded loads: column of k-slice q in step s is base + 4*s'... = cb + q
    {
        const int64_t c_begin = nfull * kGramCols;
        const int64_t nsteps = (d - c_begin + 3) / 4;      // steps of 4 columns (one per k-slice)
        for (int64_t s = gw; s < nsteps; s += nwaves) {
            const int64_t c = c_begin + 4 * s + q;
            float x[NB];
#pragma unroll
            for (int I = 0; I < NB; ++I) x[I] = (rowok[I] && c < d) ? rowp[I][c] : 0.0f;
            g.mac(x);
            if (++since_flush == 8 * kFlush) { g.flush(); since_flush = 0; }
        }
    }
    g.flush();

    // add the four waves in wave order, then write this workgroup's partial tiles
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int idx = t * 256 + v * 64 + lane;
                    red[idx] = (w == 0) ? g.sum[t][v] : red[idx] + g.sum[t][v];
                }
        }
        __syncthreads();
    }
    double *dst = partials + (int64_t)blockIdx.x * (NT * 256);
    for (int e = threadIdx.x; e < NT * 256; e += kGramThreads) dst[e] = red[e];
}

// Element (i, j), i >= j, of the Gram matrix inside the reduced tile array.  Tile (I, J) holds
// rows 16I.. as the A operand and rows 16J.. as the B operand; the instruction leaves entry
// (a, b) of its 16x16 result in register a%4 of lane 16*(a/4) + b.
__device__ __forceinline__ double gram_at(const double *__restrict__ reduced, int i, int j)
{
    const int I = i >> 4, J = j >> 4, a = i & 15, b = j & 15;
    const int t = I * (I + 1) / 2 + J;
    return reduced[t * 256 + (a & 3) * 64 + 16 * (a >> 2) + b];
}

__global__ void finalize_gram_kernel(const double *__restrict__ reduced, int n,
                                     double *__restrict__ dist, int accumulate)
{
    for (int e = threadIdx.x; e < n * n; e += blockDim.x) {
        const int i = e / n, j = e % n;
        const int hi = i > j ? i : j, lo = i > j ? j : i;
        double v = 0.0;
        if (hi != lo) {
            v = (gram_at(reduced, hi, hi) + gram_at(reduced, lo, lo)) - 2.0 * gram_at(reduced, hi, lo);
            v = v < 0.0 ? 0.0 : v;
        }
        dist[e] = accumulate ? dist[e] + v : v;
    }
}

// ------------------------------------------------------------------ reduce
// reduced[e] = sum over workgroups b of partials[b][e], added in a fixed order: 16 contiguous
// segments of workgroups are summed independently, then the 16 segment sums are added in order.
__global__ __launch_bounds__(1024) void reduce_partials_kernel(const double *__restrict__ partials,
                                                               int nblocks, int stride, int slots,
                                                               double *__restrict__ reduced)
{
    __shared__ double seg_sum[16][64];
    const int el = threadIdx.x & 63;
    const int seg = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + el;
    const int per = (nblocks + 15) / 16;
    const int b0 = seg * per;
    const int b1 = (b0 + per < nblocks) ? b0 + per : nblocks;
    double s = 0.0;
    if (e < slots)
        for (int b = b0; b < b1; ++b) s += partials[(int64_t)b * stride + e];
    seg_sum[seg][el] = s;
    __syncthreads();
    if (seg == 0 && e < slots) {
        double tot = 0.0;
#pragma unroll
        for (int k = 0; k < 16; ++k) tot += seg_sum[k][el];
        reduced[e] = tot;
    }
}

}  // namespace

int dist_grid_blocks(int64_t d, int algo)
{
    // enough workgroups to fill 256 CUs several times over, few enough that the partial sums stay
    // small next to the input
    if (algo == 1) {  // direct: one tile of 128 columns per workgroup step
        const int64_t tiles = (d + kDirTile - 1) / kDirTile;
        return (int)(tiles < 1024 ? tiles : 1024);
    }
    const int64_t steps = (d + 4 * kGramCols - 1) / (4 * kGramCols);
    return (int)(steps < 1024 ? (steps < 1 ? 1 : steps) : 1024);
}

hipError_t launch_dist_direct(const float *G, int n, int64_t d, int64_t ld, double *partials,
                              int nblocks, hipStream_t s)
{
    const int nb = (n + kRB - 1) / kRB;
    const int npb = nb * (nb + 1) / 2;
    const dim3 grid(nblocks, (npb + 15) / 16);
    dist_direct_kernel<<<grid, dim3(kDirThreads), 0, s>>>(G, n, d, ld, partials, npb);
    return hipGetLastError();
}

template <int NB>
static hipError_t launch_gram_nb(const float *G, int n, int64_t d, int64_t ld, double *partials,
                                 int nblocks, hipStream_t s)
{
    const bool aligned = ((uintptr_t)G % 16 == 0) && (ld % 4 == 0);
    if (aligned)
        dist_gram_kernel<NB, true><<<dim3(nblocks), dim3(kGramThreads), 0, s>>>(G, n, d, ld, partials);
    else
        dist_gram_kernel<NB, false><<<dim3(nblocks), dim3(kGramThreads), 0, s>>>(G, n, d, ld, partials);
    return hipGetLastError();
}

hipError_t launch_dist_gram(const float *G, int n, int64_t d, int64_t ld, double *partials,
                            int nblocks, hipStream_t s)
{
    switch (gram_blocks(n)) {
        case 1: return launch_gram_nb<1>(G, n, d, ld, partials, nblocks, s);
        case 2: return launch_gram_nb<2>(G, n, d, ld, partials, nblocks, s);
        case 3: return launch_gram_nb<3>(G, n, d, ld, partials, nblocks, s);
        case 4: return launch_gram_nb<4>(G, n, d, ld, partials, nblocks, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_reduce(const double *partials, int nblocks, int stride, int slots, double *reduced,
                         hipStream_t s)
{
    reduce_partials_kernel<<<dim3((slots + 63) / 64), dim3(1024), 0, s>>>(partials, nblocks, stride, slots,
                                                                          reduced);
    return hipGetLastError();
}

hipError_t launch_finalize_direct(const double *reduced, int n, double *dist, int accumulate, hipStream_t s)
{
    finalize_direct_kernel<<<dim3(1), dim3(1024), 0, s>>>(reduced, n, dist, accumulate);
    return hipGetLastError();
}

hipError_t launch_finalize_gram(const double *reduced, int n, double *dist, int accumulate, hipStream_t s)
{
    finalize_gram_kernel<<<dim3(1), dim3(1024), 0, s>>>(reduced, n, dist, accumulate);
    return hipGetLastError();
}

}  // namespace mb
