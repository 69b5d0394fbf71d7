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
//  gram:   G = X X^T on the matrix cores (dist_gram.hip), then
//          D_ij = G_ii + G_jj - 2 G_ij in fp64 (finalize_gram_kernel here).
//
// Every workgroup writes its partial sums as doubles; a second kernel adds
// them over workgroups in index order and a third forms the n x n matrix.
#include <hip/hip_runtime.h>

#include "gram_combine.hpp"
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
            if (!(v == v)) v = __builtin_huge_val();   // a gradient that holds a NaN or an infinity is infinitely far away
        }
        dist[e] = accumulate ? dist[e] + v : v;
    }
}

// ------------------------------------------------- gram: matrix -> distances
// Every pair takes its value from the pass with the smaller error bound (gram_combine.hpp).  Rows
// that are copies of an earlier row take over that row's distances: the split-bf16 products are
// not symmetric in their operands (hi*lo and lo*hi are added at different moments), so without
// this two bit-identical rows could get distance rows that differ in the last bits, and ties
// between their scores would hang on rounding.
__global__ __launch_bounds__(1024) void finalize_gram_kernel(const double *__restrict__ reduced,
                                                             const double *__restrict__ reduced2,
                                                             const int *__restrict__ gate, int n,
                                                             double *__restrict__ dist, int accumulate)
{
    __shared__ double D[kMaxN * kMaxN];
    __shared__ int rep[kMaxN];
    const bool refined = gate && gate[kGateFlag] != 0;
    if ((int)threadIdx.x < kMaxN) rep[threadIdx.x] = threadIdx.x;
    __syncthreads();
    for (int e = threadIdx.x; e < n * n; e += blockDim.x) {
        const int i = e / n, j = e % n;
        if (i > j && gram_term(reduced, i, j).same) atomicMin(&rep[i], j);   // the first row that i copies
    }
    __syncthreads();
    for (int e = threadIdx.x; e < n * n; e += blockDim.x) {
        const int i = rep[e / n], j = rep[e % n];
        double v = i == j ? 0.0 : gram_pair_distance(reduced, reduced2, refined, i > j ? i : j, i > j ? j : i);
        if (!(v == v)) v = __builtin_huge_val();   // a gradient that holds a NaN or an infinity is infinitely far away
        dist[e] = accumulate ? dist[e] + v : v;
    }
}

// ------------------------------------------------------------------ reduce
// reduced[e] = sum over workgroups b of partials[b][e], added in a fixed order: kRedSegs contiguous
// segments of workgroups are summed independently, then the segment sums are added in order.  A
// workgroup takes kRedSlots consecutive entries (128 contiguous bytes per partial tile) so that the
// launch has many workgroups and every thread only a few loads, all in flight at once: the kernel
// is a chain of memory latencies, not of bytes.
constexpr int kRedSegs = 64;
constexpr int kRedSlots = 16;
constexpr int kRedBatch = 16;

__global__ __launch_bounds__(kRedSegs * kRedSlots) void reduce_partials_kernel(
    const double *__restrict__ partials, int nblocks, int stride, int slots, double *__restrict__ reduced,
    int *__restrict__ ticket)
{
    __shared__ double seg_sum[kRedSegs][kRedSlots + 1];
    if (ticket && blockIdx.x == 0 && threadIdx.x == 0) *ticket = 0;   // for the launch that follows in the stream
    const int el = threadIdx.x % kRedSlots;
    const int seg = threadIdx.x / kRedSlots;
    const int e = blockIdx.x * kRedSlots + el;
    const int per = (nblocks + kRedSegs - 1) / kRedSegs;
    const int b0 = seg * per;
    const int b1 = (b0 + per < nblocks) ? b0 + per : nblocks;
    double s = 0.0;
    if (e < slots) {
        for (int b = b0; b < b1; b += kRedBatch) {
            double x[kRedBatch];
#pragma unroll
            for (int k = 0; k < kRedBatch; ++k)
                x[k] = (b + k < b1) ? partials[(int64_t)(b + k) * stride + e] : 0.0;
#pragma unroll
            for (int k = 0; k < kRedBatch; ++k) s += x[k];
        }
    }
    seg_sum[seg][el] = s;
    __syncthreads();
    if (seg == 0 && e < slots) {
        double tot = 0.0;
#pragma unroll 8
        for (int k = 0; k < kRedSegs; ++k) tot += seg_sum[k][el];
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
    const int64_t steps = (d + 127) / 128;   // one step of 32 columns for each of 4 waves
    return (int)(steps < kGramMaxBlocks ? (steps < 1 ? 1 : steps) : kGramMaxBlocks);
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

hipError_t launch_reduce(const double *partials, int nblocks, int stride, int slots, double *reduced,
                         int *ticket, hipStream_t s)
{
    reduce_partials_kernel<<<dim3((slots + kRedSlots - 1) / kRedSlots), dim3(kRedSegs * kRedSlots), 0, s>>>(
        partials, nblocks, stride, slots, reduced, ticket);
    return hipGetLastError();
}

hipError_t launch_finalize_direct(const double *reduced, int n, double *dist, int accumulate, hipStream_t s)
{
    finalize_direct_kernel<<<dim3(1), dim3(1024), 0, s>>>(reduced, n, dist, accumulate);
    return hipGetLastError();
}

hipError_t launch_finalize_gram(const double *reduced, const double *reduced2, const int *gate, int n, double *dist,
                                int accumulate, hipStream_t s)
{
    finalize_gram_kernel<<<dim3(1), dim3(1024), 0, s>>>(reduced, reduced2, gate, n, dist, accumulate ? 1 : 0);
    return hipGetLastError();
}

}  // namespace mb
