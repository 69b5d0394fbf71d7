// Distance pass, Gram form on the matrix cores (Algorithm 1, multi-Krum, the score line; Eq. 4):
// G = X X^T accumulated over all coordinates, D_ij = G_ii + G_jj - 2 G_ij afterwards in fp64.
//
// Rows are padded to NB = ceil(n/16) blocks of 16 and only the lower block triangle of G is
// computed: NT = NB(NB+1)/2 tiles of 16x16.  In a step of 32 columns lane (r = lane%16,
// q = lane/16) holds the 8 values of row 16I+r at columns 8q..8q+7 for every row block I:
// exactly the operand layout of the MFMA instructions (row = lane%16, k group = lane/16), and
// the A and B operands of a Gram product share it, so tile (I,J) is mfma(x[I], x[J]).
//
// Two kernels, which differ in how the operands arrive:
//  gram_dma_kernel  rows that start on 16-byte boundaries: tiles of 512 bytes per row go from HBM
//                   straight into LDS (described at the kernel); also takes bf16 input.
//  gram_kernel      any alignment and stride: a wave owns steps of 32 columns, walked grid-strided
//                   so that neighbouring waves read neighbouring 128-byte lines of every row; the
//                   lane loads its 32 bytes itself, DEPTH steps ahead in a register ring; nothing
//                   is staged in LDS and the main loop has no data-dependent barrier.
//
// Two arithmetic variants:
//  fp32:  v_mfma_f32_16x16x4_f32, eight k-slices per step.  At n = 39 its 1536 MACs per
//         coordinate take exactly as long as the 156 bytes take from HBM: on the ridge.
//  bf16:  every fp32 value is split exactly into three bf16 pieces x = hi + mid + lo (8
//         significand bits each, each the remainder so far rounded to nearest, so the
//         remainders are exact; seven vector instructions for two values).  A product x*y is the sum of nine piece products, each exact
//         in fp32; the six largest (hi*hi, hi*mid, mid*hi, hi*lo, lo*hi, mid*mid) are
//         accumulated, the dropped ones (mid*lo, lo*mid, lo*lo) are below 2^-26 of x*y each and
//         of either sign from one coordinate to the next.  v_mfma_f32_16x16x32_bf16 consumes a whole step
//         per instruction: six of them at 16 cycles replace eight at 32, so the matrix cores
//         stop being the limit and the kernel is bound by the HBM stream.
//
// Precision: the MFMA accumulators are fp32; every 256 columns of a wave they are handed over to
// fp64 sums (gram_kernel: the four waves of a workgroup through LDS, each thread adding its share
// in wave order; gram_dma_kernel: each wave its own, the waves adding up in order at the end).
// Workgroup sums are written as fp64 partial tiles and added over workgroups in index
// order by reduce_partials_kernel.  No atomics: the result is a function of the data only.
#include <hip/hip_runtime.h>

#include <mutex>

#include "gram_combine.hpp"
#include "mb_internal.hpp"

namespace mb {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;  // 4 waves
constexpr int kCols = 32;      // columns per wave step
constexpr int kFlush = 8;      // steps between hand-overs of the fp32 accumulators to fp64

struct Pieces {
    uintx4 hi, mid, lo;   // 8 bf16 each: element e in half (e & 1) of word e / 2
};

// two floats -> one packed bf16 pair, rounded to nearest even (v_cvt_pk_bf16_f32): a in the lower half
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16(float a, float b)
{
    const floatx2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// x minus one half of a packed bf16 pair, in one instruction: v_dot2c_f32_bf16 adds the two
// products of its bf16 pairs to x, and the second pair is (-1, 0) or (0, -1).  The result is exact
// wherever the subtraction is (checked against it bit for bit on 2e9 random pairs, both levels of
// the split).  The selecting pairs are handed over in scalar registers and kept opaque to the
// compiler: written as immediates they would be encoded as inline constants, which this
// instruction reads as fp32 words, i.e. with the -1 in the upper half either way.
struct HalfSel {
    unsigned lo, hi;   // selects the lower / the upper half of the pair
};
__device__ __forceinline__ HalfSel half_sel()
{
    unsigned lo = 0x0000bf80u, hi = 0xbf800000u;
    asm volatile("" : "+s"(lo), "+s"(hi));
    return HalfSel{lo, hi};
}
__device__ __forceinline__ float minus_half(float x, unsigned pair, unsigned sel)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, sel), x, false);
}

// two floats -> one packed word of each piece.  Every piece is the remainder so far rounded to
// nearest, so the remainders are exact, of either sign, and at most half an ulp of the piece
// before: |mid| <= 2^-9 |x|, |lo| <= 2^-18 |x|, and lo has at most 7 significant bits left.
// (Truncation would do as well for exactness, but its remainders all carry the sign of x: the
// dropped products mid*lo then have the sign of x_i*x_j in every coordinate and add up to a
// bias of about 6e-8 of |G_ij|, i.e. 1.2e-7 of the norms in the distance of two rows that point in
// opposite directions.)  Seven instructions for two values.
__device__ __forceinline__ void split_pair(float a, float b, const HalfSel &hs, unsigned &hi, unsigned &mid,
                                           unsigned &lo)
{
    hi = pack_bf16(a, b);
    const float ra = minus_half(a, hi, hs.lo);
    const float rb = minus_half(b, hi, hs.hi);
    mid = pack_bf16(ra, rb);
    const float sa = minus_half(ra, mid, hs.lo);
    const float sb = minus_half(rb, mid, hs.hi);
    lo = pack_bf16(sa, sb);
}

__device__ __forceinline__ Pieces split8(const float4 &u, const float4 &w, const HalfSel &hs)
{
    unsigned h[4], m[4], l[4];
    split_pair(u.x, u.y, hs, h[0], m[0], l[0]);
    split_pair(u.z, u.w, hs, h[1], m[1], l[1]);
    split_pair(w.x, w.y, hs, h[2], m[2], l[2]);
    split_pair(w.z, w.w, hs, h[3], m[3], l[3]);
    Pieces p;
    p.hi = uintx4{h[0], h[1], h[2], h[3]};
    p.mid = uintx4{m[0], m[1], m[2], m[3]};
    p.lo = uintx4{l[0], l[1], l[2], l[3]};
    return p;
}

struct Raw {
    float4 u, w;   // columns 8q..8q+3 and 8q+4..8q+7 of one row
};

__device__ __forceinline__ Raw raw_minus(const Raw &a, const Raw &b)
{
    Raw y;
    y.u = make_float4(a.u.x - b.u.x, a.u.y - b.u.y, a.u.z - b.u.z, a.u.w - b.u.w);
    y.w = make_float4(a.w.x - b.w.x, a.w.y - b.w.y, a.w.z - b.w.z, a.w.w - b.w.w);
    return y;
}

template <int NB>
struct Tiles {
    static constexpr int NT = NB * (NB + 1) / 2;
    floatx4 acc[NT];

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // fp32 variant: eight k-slices, slice e = element e of every lane
    __device__ __forceinline__ void mac_fp32(const Raw (&x)[NB])
    {
#define MB_SLICE(FIELD)                                                                          \
    {                                                                                            \
        int t = 0;                                                                               \
        _Pragma("unroll") for (int I = 0; I < NB; ++I)                                           \
            _Pragma("unroll") for (int J = 0; J <= I; ++J, ++t)                                  \
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[I].FIELD, x[J].FIELD, acc[t], 0, 0, 0); \
    }
        MB_SLICE(u.x) MB_SLICE(u.y) MB_SLICE(u.z) MB_SLICE(u.w)
        MB_SLICE(w.x) MB_SLICE(w.y) MB_SLICE(w.z) MB_SLICE(w.w)
#undef MB_SLICE
    }

    // bf16 input: u and w hold the raw bf16 values of two 32-column steps
    __device__ __forceinline__ void mac_in16(const Raw (&x)[NB])
    {
#define MB_STEP(FIELD)                                                                          \
    {                                                                                           \
        int t = 0;                                                                              \
        _Pragma("unroll") for (int I = 0; I < NB; ++I)                                          \
            _Pragma("unroll") for (int J = 0; J <= I; ++J, ++t)                                 \
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                               \
                    __builtin_bit_cast(bf16x8, x[I].FIELD), __builtin_bit_cast(bf16x8, x[J].FIELD), \
                    acc[t], 0, 0, 0);                                                           \
    }
        MB_STEP(u) MB_STEP(w)
#undef MB_STEP
    }

    // fp16 input: the same with the fp16 instruction (a product of two fp16 values is exact in fp32 too)
    __device__ __forceinline__ void mac_inf16(const Raw (&x)[NB])
    {
#define MB_STEP(FIELD)                                                                          \
    {                                                                                           \
        int t = 0;                                                                              \
        _Pragma("unroll") for (int I = 0; I < NB; ++I)                                          \
            _Pragma("unroll") for (int J = 0; J <= I; ++J, ++t)                                 \
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(                                \
                    __builtin_bit_cast(halfx8, x[I].FIELD), __builtin_bit_cast(halfx8, x[J].FIELD), \
                    acc[t], 0, 0, 0);                                                           \
    }
        MB_STEP(u) MB_STEP(w)
#undef MB_STEP
    }

    // bf16 variant: six piece products, the small ones first
    __device__ __forceinline__ void mac_bf16(const Pieces (&x)[NB])
    {
#define MB_TERM(PA, PB)                                                                        \
    {                                                                                          \
        int t = 0;                                                                             \
        _Pragma("unroll") for (int I = 0; I < NB; ++I)                                         \
            _Pragma("unroll") for (int J = 0; J <= I; ++J, ++t)                                \
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(                              \
                    __builtin_bit_cast(bf16x8, x[I].PA), __builtin_bit_cast(bf16x8, x[J].PB),  \
                    acc[t], 0, 0, 0);                                                          \
    }
        MB_TERM(lo, hi) MB_TERM(hi, lo) MB_TERM(mid, mid) MB_TERM(mid, hi) MB_TERM(hi, mid) MB_TERM(hi, hi)
#undef MB_TERM
    }
};

// ---------------------------------------------------------------------------------------------
// The second, centred pass (see gram_combine.hpp for why and when).  Its kernels are the two below
// with CENTER set: every workgroup first decides from the first pass's Gram tiles whether the pass
// is needed at all and which row is the pivot (the same arithmetic on the same data in every
// workgroup, so they all agree; an unneeded pass costs a launch of workgroups that read n^2/2 Gram
// entries and return), workgroup 0 leaves flag and pivot for the kernels that follow, and the
// pivot's value is subtracted from every value of its column before the products are formed.
//
// gram_gate: every thread of the workgroup calls it (barriers inside).  `scratch`: LDS, n*n + n
// doubles and two ints.  Returns the pivot row if some pair of the first pass is flagged, else -1.
template <int NTHREADS>
__device__ __forceinline__ int gram_gate(const double *__restrict__ R1, int n, double *scratch, int tid)
{
    bool bad = false;
    for (int e = tid; e < n * n; e += NTHREADS) {
        const int i = e / n, j = e % n;
        if (i > j) bad = bad || gram_flagged(gram_term(R1, i, j));
    }
    if (!__syncthreads_or(bad ? 1 : 0)) return -1;
    // pivot: the row whose k-th nearest other row is nearest, k = half of the others
    double *D = scratch, *radius = scratch + n * n;
    int *pick = reinterpret_cast<int *>(radius + n);
    const double inf = __builtin_huge_val();
    for (int e = tid; e < n * n; e += NTHREADS) {
        const int i = e / n, j = e % n;
        double v = inf;                                   // a row is not its own neighbour
        if (i != j) {
            v = gram_term(R1, i > j ? i : j, i > j ? j : i).d;
            if (!(v == v)) v = inf;
        }
        D[e] = v;
    }
    __syncthreads();
    const int k = n / 2;                                  // ceil((n - 1) / 2) of the n - 1 others
    for (int i = tid; i < n; i += NTHREADS) {
        double r = inf;
        for (int j = 0; j < n; ++j) {
            const double v = D[i * n + j];
            int before = 0;
            for (int j2 = 0; j2 < n; ++j2) {
                const double u = D[i * n + j2];
                before += (u < v || (u == v && j2 < j)) ? 1 : 0;
            }
            if (before == k - 1) r = v;
        }
        radius[i] = r;
    }
    __syncthreads();
    if (tid == 0) {
        int best = 0;
        for (int i = 1; i < n; ++i)
            if (radius[i] < radius[best]) best = i;
        *pick = best;
    }
    __syncthreads();
    return *pick;
}

// What a workgroup of the second pass does when the first pass needs no second one (so that the
// launch is not wasted): workgroup i prepares row i (and i + the grid size, ..) of the distance matrix for the selection
// kernel, which otherwise does this for all rows on one compute unit.  The row is formed exactly
// as finalize_gram_kernel and select_kernel form it from the first pass's tiles (copies of a row
// take the distances of the first of them, a NaN becomes +inf), then ordered by (distance, index)
// without the row itself: ordered[i][r] = the r-th smallest distance, idx[i][r] = that neighbour,
// idx[64*64 + 64 i + j] = the rank of neighbour j.  Every thread of the workgroup calls it;
// `scratch`: 64 doubles and 64 ints of LDS.
template <int NTHREADS>
__device__ __forceinline__ void prepare_row(const double *__restrict__ R1, int n, int i, double *scratch,
                                            double *__restrict__ ordered, unsigned char *__restrict__ idx, int tid)
{
    double *v = scratch;
    int *rep = reinterpret_cast<int *>(scratch + kMaxN);
    __syncthreads();                       // the scratch may still be read as the gate's
    if (tid < kMaxN) rep[tid] = tid;
    __syncthreads();
    for (int e = tid; e < n * n; e += NTHREADS) {
        const int a = e / n, b = e % n;
        if (a > b && gram_term(R1, a, b).same) atomicMin(&rep[a], b);
    }
    __syncthreads();
    const double inf = __builtin_huge_val();
    if (tid < n) {
        const int a = rep[i], b = rep[tid];
        double x = 0.0;
        if (a != b) x = gram_pair_distance(R1, nullptr, false, a > b ? a : b, a > b ? b : a);
        v[tid] = (x == x) ? x : inf;
    }
    __syncthreads();
    if (tid < n && tid != i) {
        const double mine = v[tid];
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const double u = v[j];
            rank += (j != i && (u < mine || (u == mine && j < tid))) ? 1 : 0;
        }
        ordered[i * kMaxN + rank] = mine;
        idx[i * kMaxN + rank] = (unsigned char)tid;
        idx[kMaxN * kMaxN + i * kMaxN + tid] = (unsigned char)rank;
    }
}

// Second pass only: the workgroup that finishes last adds up the tiles of all workgroups, in
// workgroup order (a function of the data alone), and leaves the sums where the reduction kernel
// would have put them, so that no reduction launch has to follow a pass that mostly does not run.
// Nothing waits for anything: a workgroup draws a ticket once its own tile is visible device-wide,
// and whoever draws the last one finds every tile written.  gate[kGateTicket] is 0 at the start of
// the launch (the first pass's reduction kernel, which precedes it in the stream, sets it).
// Every thread of the workgroup calls it, after its stores to `partials`; `last` is a word of LDS
// no thread still reads.  NT x 256 entries per tile set, kThreads = 256 threads.
template <int NT>
__device__ __forceinline__ void sum_tiles_if_last(const double *partials, double *__restrict__ sums, int *gate,
                                                  int *last, int tid)
{
    __threadfence();   // release: this thread's part of the tile
    __syncthreads();
    if (tid == 0) *last = (atomicAdd(&gate[kGateTicket], 1) == (int)gridDim.x - 1) ? 1 : 0;
    __syncthreads();
    if (*last == 0) return;
    __threadfence();   // acquire: the other workgroups' tiles
    const int nb = (int)gridDim.x;
    double acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = 0.0;
    constexpr int kAhead = NT <= 3 ? 8 : 4;   // workgroups whose entries are in flight together
    for (int b = 0; b < nb; b += kAhead) {
        double x[kAhead][NT];
#pragma unroll
        for (int k = 0; k < kAhead; ++k) {
            const int bb = b + k < nb ? b + k : nb - 1;
            const double *src = partials + (int64_t)bb * (NT * 256);
#pragma unroll
            for (int t = 0; t < NT; ++t) x[k][t] = src[t * 256 + tid];
        }
#pragma unroll
        for (int k = 0; k < kAhead; ++k) {
            if (b + k < nb) {
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t] += x[k][t];
            }
        }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) sums[t * 256 + tid] = acc[t];
}

template <int NB, bool BF16, int DEPTH, bool CENTER>
__global__ __launch_bounds__(kThreads) void gram_kernel(const float *__restrict__ G, int n, int64_t d,
                                                        int64_t ld, int aligned,
                                                        double *__restrict__ partials,
                                                        const double *__restrict__ first_pass,
                                                        double *__restrict__ second_sums, int *__restrict__ gate,
                                                        double *__restrict__ prep_ordered,
                                                        unsigned char *__restrict__ prep_idx)
{
    constexpr int NT = NB * (NB + 1) / 2;
    constexpr int NR = NB + (CENTER ? 1 : 0);   // row blocks a lane loads: with CENTER, the pivot row as one more
    __shared__ float stage[4][NT * 256];
    static_assert(!CENTER || sizeof(stage) >= (16 * NB * (16 * NB + 1)) * sizeof(double) + 2 * sizeof(int),
                  "the gate's scratch fits the staging area");
    const int tid = threadIdx.x;
    const HalfSel hs = half_sel();
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane & 15;   // row within a block of 16
    const int q = lane >> 4;   // group of 8 consecutive columns
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t gw = (int64_t)blockIdx.x * 4 + wave;

    int pivot = 0;
    if constexpr (CENTER) {
        pivot = gram_gate<kThreads>(first_pass, n, reinterpret_cast<double *>(&stage[0][0]), tid);
        if (blockIdx.x == 0 && tid == 0) {
            gate[kGateFlag] = pivot >= 0 ? 1 : 0;
            gate[kGatePivot] = pivot >= 0 ? pivot : 0;
        }
        if (pivot < 0) {           // the same in every thread of every workgroup
            if (prep_ordered)
                for (int row = (int)blockIdx.x; row < n; row += (int)gridDim.x)   // one row each, as a rule
                    prepare_row<kThreads>(first_pass, n, row, reinterpret_cast<double *>(&stage[0][0]), prep_ordered,
                                          prep_idx, tid);
            return;
        }
        __syncthreads();           // the scratch becomes the staging area
    }

    // Lanes of padded rows (16I + r >= n) read row n-1 instead: they fill Gram entries of rows
    // that do not exist and that nothing reads, the addresses are those another lane loads
    // anyway, and the main loop stays free of branches.
    const float *rowp[NR];
#pragma unroll
    for (int I = 0; I < NB; ++I) {
        const int row = 16 * I + r;
        rowp[I] = G + (int64_t)(row < n ? row : n - 1) * ld + 8 * q;
    }
    if constexpr (CENTER) rowp[NB] = G + (int64_t)pivot * ld + 8 * q;

    Tiles<NB> tiles;
    tiles.clear();
    double sums[NT];   // thread tid owns entry tid of every tile
#pragma unroll
    for (int t = 0; t < NT; ++t) sums[t] = 0.0;

    // hand the fp32 accumulators of the four waves over to the fp64 sums (whole workgroup)
    auto flush = [&]() {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int v = 0; v < 4; ++v) stage[wave][t * 256 + v * 64 + lane] = tiles.acc[t][v];
            tiles.acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int w = 0; w < 4; ++w) sums[t] += (double)stage[w][t * 256 + tid];
        __syncthreads();
    };

    auto load = [&](Raw (&b)[NR], int64_t step) {
        const int64_t c = step * kCols;
#pragma unroll
        for (int I = 0; I < NR; ++I) {
            b[I].u = *reinterpret_cast<const float4 *>(rowp[I] + c);
            b[I].w = *reinterpret_cast<const float4 *>(rowp[I] + c + 4);
        }
    };
    // the products of one step (with CENTER: of the values minus the pivot's)
    auto multiply = [&](const Raw (&b)[NR]) {
        Raw x[NB];
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            x[I] = b[I];
            if constexpr (CENTER) x[I] = raw_minus(b[I], b[NB]);
        }
        if constexpr (BF16) {
            Pieces p[NB];
#pragma unroll
            for (int I = 0; I < NB; ++I) p[I] = split8(x[I].u, x[I].w, hs);
            tiles.mac_bf16(p);
        } else {
            tiles.mac_fp32(x);
        }
    };

    // ---- main part: every wave of the grid runs the same number of whole steps -------------
    const int64_t nfull = aligned ? d / kCols : 0;   // steps of 32 whole columns, 16-byte loads
    const int64_t iters = nfull / nwaves;            // step gw + i*nwaves exists for all i < iters
    if (iters > 0) {
        const int64_t last = iters - 1;
        auto step_of = [&](int64_t i) { return gw + (i < last ? i : last) * nwaves; };  // clamped
        Raw raw[DEPTH][NR];
#pragma unroll
        for (int k = 0; k < DEPTH; ++k) load(raw[k], step_of(k));
        for (int64_t i = 0; i <= last; i += DEPTH) {
#pragma unroll
            for (int k = 0; k < DEPTH; ++k) {
                if (i + k <= last) {
                    if constexpr (BF16) {
                        Raw cur[NR];
#pragma unroll
                        for (int I = 0; I < NR; ++I) cur[I] = raw[k][I];
                        load(raw[k], step_of(i + k + DEPTH));
                        multiply(cur);
                    } else {
                        multiply(raw[k]);
                        load(raw[k], step_of(i + k + DEPTH));
                    }
                    if (((i + k) & (kFlush - 1)) == kFlush - 1) flush();
                }
            }
        }
    }

    // ---- what is left: fewer than one step per wave, or everything when the matrix is not
    //      16-byte aligned; element loads guarded against the end of the row --------------------
    {
        const int64_t c_begin = iters * nwaves * kCols;
        const int64_t tsteps = (d - c_begin + kCols - 1) / kCols;
        const int64_t first = (int64_t)blockIdx.x * 4;
        const int64_t titers = first < tsteps ? (tsteps - first + nwaves - 1) / nwaves : 0;  // same for 4 waves
        for (int64_t i = 0; i < titers; ++i) {
            const int64_t step = gw + i * nwaves;
            if (step < tsteps) {
                const int64_t c = c_begin + step * kCols;     // rowp already holds + 8q
                Raw x[NR];
#pragma unroll
                for (int I = 0; I < NR; ++I) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = (c + 8 * q + e < d) ? rowp[I][c + e] : 0.0f;
                    x[I].u = make_float4(v[0], v[1], v[2], v[3]);
                    x[I].w = make_float4(v[4], v[5], v[6], v[7]);
                }
                multiply(x);
            }
            if ((i & (kFlush - 1)) == kFlush - 1) flush();
        }
    }
    flush();

    double *dst = partials + (int64_t)blockIdx.x * (NT * 256);
#pragma unroll
    for (int t = 0; t < NT; ++t) dst[t * 256 + tid] = sums[t];
    if constexpr (CENTER) {
        __syncthreads();   // the staging area is free
        sum_tiles_if_last<NT>(partials, second_sums, gate, reinterpret_cast<int *>(&stage[0][0]), tid);
    }
}

// ---------------------------------------------------------------------------------------------
// The same computation with the tiles brought into LDS by the memory pipeline itself
// (global_load_lds_dwordx4); used when the matrix is 16-byte aligned.
//
// A workgroup of four waves takes tiles of 128 columns: n rows of 512 contiguous bytes.  One load
// instruction moves two such rows (half a wave each) straight into LDS, 16 bytes per lane, with
// the non-temporal hint.  No registers hold data in flight, so kStages - 1 whole tiles per
// workgroup are on their way while one is multiplied, and three workgroups fit a compute unit.
// Row-contiguous non-temporal requests of this size stream at 7.1 TB/s here, against 6.2 TB/s
// for the operand-layout loads of the kernel above.
//
// LDS layout of a tile: row i at byte 512 i; the 16-byte chunk c of a row sits in slot
// c ^ (i & 15).  A direct load puts lane l's 16 bytes at (base + 16 l), so the swizzle costs
// nothing: lane l simply fetches the chunk that belongs in its slot.  Wave w then reads columns
// 32w..32w+31 of every row in the operand layout (lane (r, q): chunks 8w+2q and 8w+2q+1 of rows
// 16I + r); the 16 rows that one quarter of the wave reads sit in 16 different slots, so the
// 16-byte LDS reads have no bank conflicts.
//
// Synchronisation per tile: every wave waits until its own loads of the tile have landed
// (s_waitcnt vmcnt, younger tiles stay in flight), one workgroup barrier, then the loads for the
// buffer that was read before the barrier are issued.  Each wave issues exactly L load
// instructions per tile so that the count to wait for is a constant: a wave whose last row pair
// does not exist fetches 16 bytes into a spare slot instead.  The LDS reads are written in
// assembly together with their wait: the compiler would otherwise place them behind a wait for
// every outstanding direct load.
//
// Each wave converts its own fp32 accumulators to fp64 every 8 tiles (256 of its columns); the
// four waves add up through LDS in wave order at the end.
constexpr int kTile = 128;   // columns per workgroup tile

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef __attribute__((address_space(1))) const void *global_void_ptr;

__device__ __forceinline__ unsigned lds_byte_address(const float *p)
{
    return (unsigned)(size_t)(__attribute__((address_space(3))) const float *)p;
}

// wait until at most N of this wave's vector-memory operations are outstanding, then the barrier
template <int N>
__device__ __forceinline__ void wait_loads_then_barrier()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// operand-layout reads of one tile: two 16-byte reads per row block, complete on return
template <int NB>
__device__ __forceinline__ void read_tile(unsigned base, const unsigned (&off)[2 * NB], Raw (&x)[NB])
{
    floatx4 v[2 * NB];
    if constexpr (NB == 1) {
        asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(v[0]), "=&v"(v[1])
                     : "v"(base + off[0]), "v"(base + off[1])
                     : "memory");
    } else if constexpr (NB == 2) {
        asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\t"
                     "ds_read_b128 %3, %7\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
                     : "v"(base + off[0]), "v"(base + off[1]), "v"(base + off[2]), "v"(base + off[3])
                     : "memory");
    } else if constexpr (NB == 3) {
        asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %7\n\tds_read_b128 %2, %8\n\t"
                     "ds_read_b128 %3, %9\n\tds_read_b128 %4, %10\n\tds_read_b128 %5, %11\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5])
                     : "v"(base + off[0]), "v"(base + off[1]), "v"(base + off[2]), "v"(base + off[3]),
                       "v"(base + off[4]), "v"(base + off[5])
                     : "memory");
    } else {
        static_assert(NB == 4, "at most 64 rows");
        asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\t"
                     "ds_read_b128 %3, %11\n\tds_read_b128 %4, %12\n\tds_read_b128 %5, %13\n\t"
                     "ds_read_b128 %6, %14\n\tds_read_b128 %7, %15\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]),
                       "=&v"(v[6]), "=&v"(v[7])
                     : "v"(base + off[0]), "v"(base + off[1]), "v"(base + off[2]), "v"(base + off[3]),
                       "v"(base + off[4]), "v"(base + off[5]), "v"(base + off[6]), "v"(base + off[7])
                     : "memory");
    }
#pragma unroll
    for (int I = 0; I < NB; ++I) {
        x[I].u = make_float4(v[2 * I][0], v[2 * I][1], v[2 * I][2], v[2 * I][3]);
        x[I].w = make_float4(v[2 * I + 1][0], v[2 * I + 1][1], v[2 * I + 1][2], v[2 * I + 1][3]);
    }
}

// the same for the pivot row alone: its two chunks, complete on return
__device__ __forceinline__ void read_pivot(unsigned base, const unsigned (&off)[2], Raw &x)
{
    floatx4 v0, v1;
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(v0), "=&v"(v1)
                 : "v"(base + off[0]), "v"(base + off[1])
                 : "memory");
    x.u = make_float4(v0[0], v0[1], v0[2], v0[3]);
    x.w = make_float4(v1[0], v1[1], v1[2], v1[3]);
}

// eight 16-bit values (four words, element e in half e & 1 of word e / 2) widened to fp32
template <int FMT>
__device__ __forceinline__ Raw widen8(const float4 &w)
{
    const unsigned a = __float_as_uint(w.x), b = __float_as_uint(w.y), c = __float_as_uint(w.z),
                   e = __float_as_uint(w.w);
    Raw y;
    y.u = make_float4(widen16<FMT>(a, false), widen16<FMT>(a, true), widen16<FMT>(b, false), widen16<FMT>(b, true));
    y.w = make_float4(widen16<FMT>(c, false), widen16<FMT>(c, true), widen16<FMT>(e, false), widen16<FMT>(e, true));
    return y;
}

// Tile buffers per workgroup and workgroups per compute unit the registers are budgeted for
// (measured at n = 39: 2 buffers x 3 workgroups 5.97 ms, 3 x 2 6.4 ms; the fp64 sums of
// 10 tiles leave room for two waves per SIMD only at NB = 4).
// Four row blocks (n > 48) leave room for two workgroups per compute unit whatever the stage count
// (236 registers), so there a third tile buffer buys a second tile in flight per workgroup for as
// long as two workgroups' buffers fit the 160 KB of LDS (n <= 52).
constexpr int kStages = 2;
constexpr int kStagesWide = 3;
constexpr int kWideMaxN = 52;
constexpr int dma_stages(int nb, int n) { return (nb == 4 && n <= kWideMaxN) ? kStagesWide : kStages; }
template <int NB>
struct DmaShape {
    static constexpr int min_blocks = NB == 4 ? 2 : 3;
};

inline int dma_pairs(int n) { return (n + 1) / 2; }   // load instructions per tile, 1 KB of LDS each
// LDS bytes of one workgroup: the tile buffers and the spare slot
inline size_t dma_lds_bytes(int n, int stages) { return (size_t)stages * dma_pairs(n) * 1024 + 1024; }

// What the kernel reads and how it multiplies:
//   kFp32    fp32 input, fp32 MFMA
//   kSplit   fp32 input, every value split into three bf16 pieces (see the top of this file)
//   kIn16    bf16 input (raw 16-bit words): products of two bf16 values are exact in fp32, one
//            v_mfma_f32_16x16x32_bf16 per tile and 32 columns, nothing to split
//   kInF16   fp16 input: the same with v_mfma_f32_16x16x32_f16
// A tile is 512 bytes of every row either way: 128 fp32 or 256 16-bit columns.
enum Kind { kFp32 = 0, kSplit = 1, kIn16 = 2, kInF16 = 3 };
template <int KIND> constexpr bool is_16bit() { return KIND == kIn16 || KIND == kInF16; }
template <int KIND> constexpr int storage_of() { return KIND == kIn16 ? kStoreBf16 : KIND == kInF16 ? kStoreFp16 : kStoreFp32; }
template <int KIND> constexpr int elem_bytes() { return is_16bit<KIND>() ? 2 : 4; }
template <int KIND> constexpr int tile_cols() { return 512 / elem_bytes<KIND>(); }

template <int NB, int KIND, int L, bool CENTER, int S>
__global__ __launch_bounds__(kThreads, DmaShape<NB>::min_blocks) void gram_dma_kernel(
    const void *__restrict__ Gv, int n, int64_t d, int64_t ld, int64_t ntiles, double *__restrict__ partials,
    const double *__restrict__ first_pass, double *__restrict__ second_sums, int *__restrict__ gate,
    double *__restrict__ prep_ordered, unsigned char *__restrict__ prep_idx)
{
    constexpr int NT = NB * (NB + 1) / 2;
    constexpr int EB = elem_bytes<KIND>();
    constexpr int TC = tile_cols<KIND>();
    constexpr int WC = TC / 4;                    // columns of a tile that one wave multiplies
    constexpr int kEvery = kFlush * 32 / WC;      // tiles between hand-overs: 256 columns of a wave
    static_assert(S >= 2 && L * (S - 2) < 64, "stage count");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const char *G = static_cast<const char *>(Gv);
    const int tid = threadIdx.x;
    const HalfSel hs = half_sel();
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane & 15;
    const int q = lane >> 4;
    const int tile_floats = ((n + 1) >> 1) * 256;

    // second pass: needed at all, and around which row?  (the tile buffers serve as scratch: n KB
    // and more, the gate needs (n^2 + n) doubles)
    int pivot = 0;
    if constexpr (CENTER) {
        pivot = gram_gate<kThreads>(first_pass, n, reinterpret_cast<double *>(lds), tid);
        if (blockIdx.x == 0 && tid == 0) {
            gate[kGateFlag] = pivot >= 0 ? 1 : 0;
            gate[kGatePivot] = pivot >= 0 ? pivot : 0;
        }
        if (pivot < 0) {           // the same in every thread of every workgroup
            if (prep_ordered)
                for (int row = (int)blockIdx.x; row < n; row += (int)gridDim.x)   // one row each, as a rule
                    prepare_row<kThreads>(first_pass, n, row, reinterpret_cast<double *>(lds), prep_ordered, prep_idx,
                                          tid);
            return;
        }
        __syncthreads();           // the scratch becomes the tile buffers
    }

    // ---- loads: instruction j of this wave moves row pair wave + 4j ---------------------------
    const int half = lane >> 5, slot = lane & 31;
    const char *src[L];
    int dst[L], dstep[L];   // float offset of the target in buffer 0, its step per buffer (same for the wave)
    bool on[L];
#pragma unroll
    for (int j = 0; j < L; ++j) {
        const int p = wave + 4 * j;
        const int row = 2 * p + half;
        if (2 * p < n) {
            on[j] = row < n;
            src[j] = G + (int64_t)(on[j] ? row : 0) * ld * EB + 16 * (slot ^ (row & 15));
            dst[j] = p * 256;
            dstep[j] = tile_floats;
        } else {   // no such rows: one lane fetches 16 bytes into the spare slot, nothing reads them
            on[j] = lane == 0;
            src[j] = G;
            dst[j] = S * tile_floats;
            dstep[j] = 0;
        }
    }
    auto issue = [&](int buf, int64_t tile) {
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (on[j])
                __builtin_amdgcn_global_load_lds((global_void_ptr)(src[j] + tile * 512),
                                                 (lds_void_ptr)(lds + dst[j] + buf * dstep[j]), 16, 0,
                                                 2 /* non-temporal */);
        }
    };

    // ---- reads: byte offsets of this lane's two chunks per row block (padded rows re-read row n-1)
    // fp32: the 8 values of one 32-column step are chunks 8w+2q and 8w+2q+1;
    // 16-bit input: a chunk is the 8 values of one step, the wave's two steps are chunks 8w+q and 8w+4+q.
    unsigned off[2 * NB];
#pragma unroll
    for (int I = 0; I < NB; ++I) {
        int row = 16 * I + r;
        row = row < n ? row : n - 1;
        const int c0 = (is_16bit<KIND>() ? 8 * wave + q : 8 * wave + 2 * q) ^ (row & 15);
        off[2 * I] = (unsigned)(row * 512 + c0 * 16);
        off[2 * I + 1] = (unsigned)(row * 512 + (c0 ^ (is_16bit<KIND>() ? 4 : 1)) * 16);
    }
    unsigned poff[2] = {0u, 0u};   // the same two chunks of the pivot row
    if constexpr (CENTER) {
        const int c0 = (is_16bit<KIND>() ? 8 * wave + q : 8 * wave + 2 * q) ^ (pivot & 15);
        poff[0] = (unsigned)(pivot * 512 + c0 * 16);
        poff[1] = (unsigned)(pivot * 512 + (c0 ^ (is_16bit<KIND>() ? 4 : 1)) * 16);
    }
    const unsigned lds0 = lds_byte_address(lds);

    Tiles<NB> tiles;
    tiles.clear();
    double sums[NT][4];   // this wave's share, accumulator layout
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) sums[t][v] = 0.0;
    auto flush = [&]() {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
            for (int v = 0; v < 4; ++v) sums[t][v] += (double)tiles.acc[t][v];
            tiles.acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto multiply = [&](const Raw (&x)[NB]) {
        if constexpr (KIND == kSplit) {
            Pieces p[NB];
#pragma unroll
            for (int I = 0; I < NB; ++I) p[I] = split8(x[I].u, x[I].w, hs);
            tiles.mac_bf16(p);
        } else if constexpr (KIND == kIn16) {
            tiles.mac_in16(x);
        } else if constexpr (KIND == kInF16) {
            tiles.mac_inf16(x);
        } else {
            tiles.mac_fp32(x);
        }
    };
    // second pass: the pivot's values come off first.  fp32 input: one subtraction per value, then
    // as above.  bf16 input: the differences of two bf16 values are fp32 values (exact when the
    // exponents are within 16 of each other), so each of the wave's two steps is widened,
    // centred and multiplied as split fp32.
    auto multiply_centred = [&](const Raw (&x)[NB], const Raw &pv) {
        if constexpr (is_16bit<KIND>()) {
            constexpr int FMT = storage_of<KIND>();
            const Raw p0 = widen8<FMT>(pv.u), p1 = widen8<FMT>(pv.w);
            Pieces p[NB];
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                const Raw y = raw_minus(widen8<FMT>(x[I].u), p0);
                p[I] = split8(y.u, y.w, hs);
            }
            tiles.mac_bf16(p);
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                const Raw y = raw_minus(widen8<FMT>(x[I].w), p1);
                p[I] = split8(y.u, y.w, hs);
            }
            tiles.mac_bf16(p);
        } else {
            Raw y[NB];
#pragma unroll
            for (int I = 0; I < NB; ++I) y[I] = raw_minus(x[I], pv);
            multiply(y);
        }
    };

    // ---- whole tiles b, b + g, b + 2g, ... of this workgroup ----------------------------------
    const int64_t g = gridDim.x, b = blockIdx.x;
    const int64_t mine = b < ntiles ? (ntiles - b + g - 1) / g : 0;
#pragma unroll
    for (int k = 0; k < S - 1; ++k)
        if (k < mine) issue(k, b + k * g);
    for (int64_t i = 0; i < mine; ++i) {
        // younger tiles in flight: min(S - 2, mine - 1 - i), L loads each
        // a wave that is ready for the next tile goes first: the sooner all four are through the
        // barrier, the sooner the next loads are on their way (measured: 1 % on the whole pass
        // where there is arithmetic to compete with, nothing with bf16 input)
        if constexpr (!is_16bit<KIND>()) __builtin_amdgcn_s_setprio(3);
        if (mine - 1 - i >= S - 2) {
            wait_loads_then_barrier<L * (S - 2)>();
        } else {
            wait_loads_then_barrier<0>();
        }
        // every wave has left the buffer of tile i - 1: refill it
        if (i + S - 1 < mine) issue((int)((i + S - 1) % S), b + (i + S - 1) * g);
        if constexpr (!is_16bit<KIND>()) __builtin_amdgcn_s_setprio(0);
        Raw x[NB];
        read_tile<NB>(lds0 + (unsigned)((int)(i % S) * tile_floats * 4), off, x);
        if constexpr (CENTER) {
            Raw pv;
            read_pivot(lds0 + (unsigned)((int)(i % S) * tile_floats * 4), poff, pv);
            multiply_centred(x, pv);
        } else {
            multiply(x);
        }
        if ((i & (kEvery - 1)) == kEvery - 1) flush();
    }

    // ---- the columns after the whole tiles: element loads, a wave takes WC columns at a time,
    //      all waves of the grid in turn (everything, when the rows are not 16-byte aligned and
    //      ntiles = 0) --------------------------------------------------------------------------
    {
        const int64_t c_begin = ntiles * TC;
        const int64_t units = (d - c_begin + WC - 1) / WC;
        const int64_t nwaves = g * 4, gw = b * 4 + wave;
        int64_t done = 0;
        for (int64_t u = gw; u < units; u += nwaves, ++done) {
            const int64_t c = c_begin + u * WC + 8 * q;      // this lane's 8 columns of the first step
            // the lane's values of one row (16-bit input: two steps, the words as they are)
            auto load_row = [&](int row) {
                Raw y;
                if constexpr (is_16bit<KIND>()) {
                    const unsigned short *p = reinterpret_cast<const unsigned short *>(G) + (int64_t)row * ld;
                    unsigned w0[4], w1[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int64_t ca = c + 2 * e, cb = c + 32 + 2 * e;
                        w0[e] = (ca < d ? (unsigned)p[ca] : 0u) | (ca + 1 < d ? (unsigned)p[ca + 1] << 16 : 0u);
                        w1[e] = (cb < d ? (unsigned)p[cb] : 0u) | (cb + 1 < d ? (unsigned)p[cb + 1] << 16 : 0u);
                    }
                    y.u = make_float4(__uint_as_float(w0[0]), __uint_as_float(w0[1]), __uint_as_float(w0[2]),
                                      __uint_as_float(w0[3]));
                    y.w = make_float4(__uint_as_float(w1[0]), __uint_as_float(w1[1]), __uint_as_float(w1[2]),
                                      __uint_as_float(w1[3]));
                } else {
                    const float *p = reinterpret_cast<const float *>(G) + (int64_t)row * ld;
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = (c + e < d) ? p[c + e] : 0.0f;
                    y.u = make_float4(v[0], v[1], v[2], v[3]);
                    y.w = make_float4(v[4], v[5], v[6], v[7]);
                }
                return y;
            };
            Raw x[NB];
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                int row = 16 * I + r;
                row = row < n ? row : n - 1;
                x[I] = load_row(row);
            }
            if constexpr (CENTER) {
                // columns past the end are zero in every row, the pivot's included: they add nothing
                multiply_centred(x, load_row(pivot));
            } else {
                multiply(x);
            }
            if ((done & (kEvery - 1)) == kEvery - 1) flush();
        }
    }
    flush();

    // ---- the four waves add up in wave order; thread tid owns entry tid of every tile ---------
    double *red = reinterpret_cast<double *>(lds);   // NT x 2 KB, less than one tile buffer pair
    double total[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) total[t] = 0.0;
    for (int w = 0; w < 4; ++w) {
        __syncthreads();
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[t * 256 + v * 64 + lane] = sums[t][v];
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < NT; ++t) total[t] += red[t * 256 + tid];
    }
    double *out = partials + (int64_t)blockIdx.x * (NT * 256);
#pragma unroll
    for (int t = 0; t < NT; ++t) out[t * 256 + tid] = total[t];
    if constexpr (CENTER) {
        __syncthreads();   // every thread has read its entries of `red`
        sum_tiles_if_last<NT>(partials, second_sums, gate, reinterpret_cast<int *>(lds), tid);
    }
}

// What the host knows about one kernel on one device: whether the LDS limit has been raised and how
// many workgroups stay resident.  Kept per device (the attribute and the occupancy are the
// device's) and behind a mutex (host threads may call concurrently).
constexpr int kMaxDevices = 64;
std::mutex g_launch_mu;

inline hipError_t current_device(int *dev)
{
    const hipError_t e = hipGetDevice(dev);
    if (e != hipSuccess) return e;
    return (*dev >= 0 && *dev < kMaxDevices) ? hipSuccess : hipErrorInvalidDevice;
}

// `second` (may be null): launch the second, centred pass instead, which reads the first pass's
// reduced Gram tiles and leaves its flag and pivot in `gate`.
struct SecondPass {
    const double *first_pass;
    double *sums;   // where its reduced tiles go
    int *gate;
    double *prep_ordered;      // may be null: rows prepared for the selection when the pass has nothing to do
    unsigned char *prep_idx;
};

template <int NB, int KIND, int L, bool CENTER, int S>
hipError_t launch_dma_s(const void *G, int n, int64_t d, int64_t ld, bool aligned, double *partials, int max_blocks,
                        int *nblocks, const SecondPass *second, hipStream_t s)
{
    struct PerDevice {
        bool prepared;
        int resident[65];   // workgroups the device holds at once, by n (LDS use grows with n)
    };
    static PerDevice cache[kMaxDevices] = {};
    hipError_t e;
    int dev = 0;
    if ((e = current_device(&dev)) != hipSuccess) return e;
    const size_t bytes = dma_lds_bytes(n, S);
    int resident = 0;
    {
        std::lock_guard<std::mutex> lock(g_launch_mu);
        PerDevice &c = cache[dev];
        if (!c.prepared) {
            if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gram_dma_kernel<NB, KIND, L, CENTER, S>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)dma_lds_bytes(S == kStagesWide ? kWideMaxN : 16 * NB, S))) != hipSuccess)
                return e;
            c.prepared = true;
        }
        if (!c.resident[n]) {
            int cus = 0, per_cu = 0;
            if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
            if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gram_dma_kernel<NB, KIND, L, CENTER, S>,
                                                                  kThreads, bytes)) != hipSuccess)
                return e;
            c.resident[n] = cus * (per_cu < 1 ? 1 : per_cu);
        }
        resident = c.resident[n];
    }
    // at least four tiles per workgroup: with fewer, writing and adding up the partial tiles costs
    // more than the distance pass itself
    constexpr int TC = tile_cols<KIND>();
    const int64_t tiles = aligned ? d / TC : 0;
    const int64_t work = aligned ? tiles : (d + TC - 1) / TC;   // element loads: a workgroup per TC columns
    int64_t g = resident < max_blocks ? resident : max_blocks;
    if (work < 4 * g) g = work < 4 ? 1 : work / 4;
    *nblocks = (int)g;
    gram_dma_kernel<NB, KIND, L, CENTER, S><<<dim3((unsigned)g), dim3(kThreads), bytes, s>>>(
        G, n, d, ld, tiles, partials, second ? second->first_pass : nullptr, second ? second->sums : nullptr,
        second ? second->gate : nullptr, second ? second->prep_ordered : nullptr,
        second ? second->prep_idx : nullptr);
    return hipGetLastError();
}

template <int NB, int KIND, int L, bool CENTER>
hipError_t launch_dma_l(const void *G, int n, int64_t d, int64_t ld, bool aligned, double *partials, int max_blocks,
                        int *nblocks, const SecondPass *second, hipStream_t s)
{
    if constexpr (NB == 4) {
        if (dma_stages(NB, n) == kStagesWide)
            return launch_dma_s<NB, KIND, L, CENTER, kStagesWide>(G, n, d, ld, aligned, partials, max_blocks, nblocks,
                                                                  second, s);
    }
    return launch_dma_s<NB, KIND, L, CENTER, kStages>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);
}

template <int NB, int KIND>
hipError_t launch_dma(const void *G, int n, int64_t d, int64_t ld, bool aligned, double *partials, int max_blocks,
                      int *nblocks, const SecondPass *second, hipStream_t s)
{
    // load instructions per wave and tile: ceil(pairs / 4), one of two values for each NB
    const bool more = (dma_pairs(n) + 3) / 4 == 2 * NB;
    if (second) {
        if (more) return launch_dma_l<NB, KIND, 2 * NB, true>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);
        return launch_dma_l<NB, KIND, 2 * NB - 1, true>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);
    }
    if (more) return launch_dma_l<NB, KIND, 2 * NB, false>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);
    return launch_dma_l<NB, KIND, 2 * NB - 1, false>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);
}

template <int NB, bool BF16, int DEPTH, bool CENTER>
hipError_t launch_one(const float *G, int n, int64_t d, int64_t ld, double *partials, int nblocks,
                      const SecondPass *second, hipStream_t s)
{
    const int aligned = ((uintptr_t)G % 16 == 0) && (ld % 4 == 0);
    gram_kernel<NB, BF16, DEPTH, CENTER><<<dim3(nblocks), dim3(kThreads), 0, s>>>(
        G, n, d, ld, aligned, partials, second ? second->first_pass : nullptr, second ? second->sums : nullptr,
        second ? second->gate : nullptr, second ? second->prep_ordered : nullptr,
        second ? second->prep_idx : nullptr);
    return hipGetLastError();
}

template <int NB, bool BF16, int DEPTH, bool CENTER>
int resident_blocks()
{
    static int cache[kMaxDevices] = {};
    int dev = 0, cus = 0, per_cu = 0;
    if (current_device(&dev) != hipSuccess) return 1024;
    std::lock_guard<std::mutex> lock(g_launch_mu);
    if (cache[dev]) return cache[dev];
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 1024;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gram_kernel<NB, BF16, DEPTH, CENTER>, kThreads, 0) !=
        hipSuccess)
        return 1024;
    if (per_cu < 1) per_cu = 1;
    cache[dev] = cus * per_cu;
    return cache[dev];
}

template <int NB, bool BF16, int DEPTH, bool CENTER>
int grid_for(int64_t d, int max_blocks)
{
    const int64_t steps = (d + 4 * kCols - 1) / (4 * kCols);   // one step for each of the 4 waves
    int64_t g = resident_blocks<NB, BF16, DEPTH, CENTER>();
    if (g > max_blocks) g = max_blocks;
    if (steps < g) g = steps < 1 ? 1 : steps;
    return (int)g;
}

// prefetch depth per variant and row-block count (register budget: 24 VGPRs per step at NB = 3)
template <int NB, bool BF16>
struct Depth {
    static constexpr int value = 4;   // measured: 1..4 within 2 % of each other at n = 39, 4 best at n = 51
};

template <int NB, bool BF16>
hipError_t launch_nb(const float *G, int n, int64_t d, int64_t ld, double *partials, int max_blocks, int *nblocks,
                     const SecondPass *second, hipStream_t s)
{
    if (((uintptr_t)G % 16 == 0) && (ld % 4 == 0) && d >= kTile)
        return launch_dma<NB, BF16 ? kSplit : kFp32>(G, n, d, ld, true, partials, max_blocks, nblocks, second, s);
    constexpr int D = Depth<NB, BF16>::value;
    if (second) {
        *nblocks = grid_for<NB, BF16, D, true>(d, max_blocks);
        return launch_one<NB, BF16, D, true>(G, n, d, ld, partials, *nblocks, second, s);
    }
    *nblocks = grid_for<NB, BF16, D, false>(d, max_blocks);
    return launch_one<NB, BF16, D, false>(G, n, d, ld, partials, *nblocks, second, s);
}

}  // namespace

hipError_t launch_dist_gram_in16(const uint16_t *G, int fmt, int n, int64_t d, int64_t ld, double *partials,
                                 int max_blocks, int *nblocks, const double *first_pass, double *second_sums,
                                 int *gate, double *prep_ordered, unsigned char *prep_idx, hipStream_t s)
{
    if (max_blocks < 1 || (fmt != kStoreBf16 && fmt != kStoreFp16)) return hipErrorInvalidValue;
    if (max_blocks > kGramMaxBlocks) max_blocks = kGramMaxBlocks;
    const SecondPass sp{first_pass, second_sums, gate, prep_ordered, prep_idx}, *second = first_pass ? &sp : nullptr;
    const bool aligned = ((uintptr_t)G % 16 == 0) && (ld % 8 == 0) && d >= tile_cols<kIn16>();
#define MB_NB(K)                                                                                                 \
    switch (gram_blocks(n)) {                                                                                    \
        case 1: return launch_dma<1, K>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);         \
        case 2: return launch_dma<2, K>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);         \
        case 3: return launch_dma<3, K>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);         \
        case 4: return launch_dma<4, K>(G, n, d, ld, aligned, partials, max_blocks, nblocks, second, s);         \
    }
    if (fmt == kStoreBf16) {
        MB_NB(kIn16)
    } else {
        MB_NB(kInF16)
    }
#undef MB_NB
    return hipErrorInvalidValue;
}

hipError_t launch_dist_gram(const float *G, int n, int64_t d, int64_t ld, double *partials, bool bf16,
                            int max_blocks, int *nblocks, const double *first_pass, double *second_sums, int *gate,
                            double *prep_ordered, unsigned char *prep_idx, hipStream_t s)
{
    if (max_blocks < 1) return hipErrorInvalidValue;
    if (max_blocks > kGramMaxBlocks) max_blocks = kGramMaxBlocks;
    const SecondPass sp{first_pass, second_sums, gate, prep_ordered, prep_idx}, *second = first_pass ? &sp : nullptr;
    const int nb = gram_blocks(n);
    if (bf16) {
        switch (nb) {
            case 1: return launch_nb<1, true>(G, n, d, ld, partials, max_blocks, nblocks, second, s);
            case 2: return launch_nb<2, true>(G, n, d, ld, partials, max_blocks, nblocks, second, s);
            case 3: return launch_nb<3, true>(G, n, d, ld, partials, max_blocks, nblocks, second, s);
            case 4: return launch_nb<4, true>(G, n, d, ld, partials, max_blocks, nblocks, second, s);
        }
    } else {
        switch (nb) {
            case 1: return launch_nb<1, false>(G, n, d, ld, partials, max_blocks, nblocks, second, s);
            case 2: return launch_nb<2, false>(G, n, d, ld, partials, max_blocks, nblocks, second, s);
            case 3: return launch_nb<3, false>(G, n, d, ld, partials, max_blocks, nblocks, second, s);
            case 4: return launch_nb<4, false>(G, n, d, ld, partials, max_blocks, nblocks, second, s);
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace mb
