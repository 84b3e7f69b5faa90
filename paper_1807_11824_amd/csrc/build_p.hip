// Alg. 1 lines 1-2 of the paper on gfx950: the sparse affinity matrix P.
//
//   row_norms            |x_i|^2 in double, rounded to float
//   split_bf16           every x as bf16 high part + bf16 low part
//   knn_tile_mfma        Sec. III-B, exact reading: all-pairs squared distances
//                        |q|^2 + |x|^2 - 2 q.x, the dot products on the matrix cores
//                        (three v_mfma_f32_32x32x16_bf16 per step on the split values, 256x128 or
//                        128x128 tiles through LDS).  The N x N matrix is never stored: the
//                        epilogue keeps a pair only if it beats the query row's current cut-off
//                        and appends it to that row's candidate buffer.
//   knn_tile_resident    the same for d <= 64 and many query rows: a workgroup keeps 256 query rows
//                        on chip for the whole launch and streams the database rows past them
//   knn_compact          per query row, sorts the buffer, keeps the best k' = k + margin and lowers
//                        the cut-off to the k'-th distance
//   knn_rerank           recomputes the k' candidate distances as sum_t (x_it - x_jt)^2 in double,
//                        orders them by (distance, index), keeps k, and certifies the row: every
//                        discarded pair had a tile distance >= cut-off, so it cannot belong to
//                        the k nearest if cut-off - error bound > exact k-th distance
//   knn_exact_dists / knn_exact_select   rows that fail the certificate: all n distances in
//                        double, radix selection of the k-th smallest, ties by index
//   ivf_probe_tiles / ivf_search_tiles   Eq. (10) and (11) of the approximate search for rows longer than 64
//                        coordinates, on the same tiles, re-rank and certificate (called from ivf.hip)
//   perplexity_search    Eq. (1) on the k neighbours, beta by bracketing + bisection on the entropy
//   sym_count / sym_fill / sym_sort_rows   p_ij = (p_j|i + p_i|j) / 2N as CSR, columns ascending
#include "tsne_internal.h"

#include <math.h>
#include <stdio.h>

namespace {

constexpr size_t ALIGN = 256;
__host__ __device__ inline size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

constexpr int QB = 65536;       // query rows per pass
constexpr int DBC = 2048;       // database rows per launch (bounds what one launch can append per row)
constexpr int MAX_KP = 1920;    // k' limit (size of the re-rank's LDS arrays)
constexpr int SORT_CAP = 4096;  // candidate buffer entries per row = LDS sort size
constexpr int TN = 128;         // database rows per tile
constexpr int KNN_MB = 4;        // 32-row query blocks per wave of the general single-level tile kernel
constexpr int COMPACT_SLACK = 64;  // new candidates per row that trigger a re-sort of its buffer
constexpr int COMPACT_EVERY = 2;   // after the resident tile kernel a compaction pass follows every second slab only (a pass
                                   // costs a third of a slab; cut-offs one slab older let a few more pairs through)
constexpr int KFLUSH = 64;      // columns summed on the matrix cores before a flush into the running sum
constexpr int HIGH_FIRST_MIN_D = 256;   // from this many columns on the exact search sweeps with the high parts first

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t orderable(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unorderable(uint32_t u)
{
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u);
}
__device__ __forceinline__ uint64_t orderable64(double d)
{
    uint64_t u = (uint64_t)__double_as_longlong(d);
    return (u & 0x8000000000000000ull) ? ~u : (u | 0x8000000000000000ull);
}

// Squared distances do not change when every row is moved by the same vector, while the error of
// the candidate search grows with the rows' norms: the search therefore works on X - mu, mu the
// column means (only the split copy and the norms are centred; the re-rank reads the caller's X).
// Any mu gives correct lists; this one is computed in a fixed order so that a build is reproducible.
constexpr int MEAN_CHUNKS = 256;     // row chunks of the first stage
__global__ __launch_bounds__(256) void col_mean_part(const float *__restrict__ X, int n, int d, int rows_per_chunk,
                                                     double *__restrict__ part)
{
    __shared__ double acc[4][64];
    const int c = blockIdx.x * 64 + (threadIdx.x & 63), rg = threadIdx.x >> 6;
    const int r0 = blockIdx.y * rows_per_chunk, r1 = min(n, r0 + rows_per_chunk);
    double s = 0.0;
    if (c < d)
        for (int r = r0 + rg; r < r1; r += 4) s += (double)X[(size_t)r * d + c];
    acc[rg][threadIdx.x & 63] = s;
    __syncthreads();
    if (rg == 0 && c < d) part[(size_t)blockIdx.y * d + c] = ((acc[0][threadIdx.x] + acc[1][threadIdx.x]) + acc[2][threadIdx.x]) + acc[3][threadIdx.x];
}

__global__ __launch_bounds__(256) void col_mean_final(const double *__restrict__ part, int nchunks, int n, int d, int dp,
                                                      float *__restrict__ mu)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= dp) return;
    double s = 0.0;
    if (c < d)
        for (int q = 0; q < nchunks; ++q) s += part[(size_t)q * d + c];
    mu[c] = c < d ? (float)(s / (double)n) : 0.f;
}

// |x - mu|^2 of the centred row as the tiles see it (each x_t - mu_t rounded to float)
// (rowmap: row r of the result is row rowmap[r] of the nsrc rows of X; null = the same rows)
__global__ __launch_bounds__(256) void row_norms(const float *__restrict__ X, const float *__restrict__ mu, int n, int d,
                                                 const int *__restrict__ rowmap, int nsrc, float *__restrict__ norms)
{
    const size_t w = global_index() >> 6;
    if (w >= (size_t)n) return;
    const int row = (int)w;
    const float *x = X + (size_t)(rowmap ? min(max(rowmap[row], 0), nsrc - 1) : row) * d;
    double s = 0.0;
    for (int t = lane_id(); t < d; t += WAVE) { double v = (double)(x[t] - mu[t]); s += v * v; }
    s = wave_sum(s);
    if (lane_id() == 0) norms[row] = (float)s;
}

__global__ void knn_reset(float *__restrict__ tau, int *__restrict__ cnt, int rows, int *__restrict__ ccount)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows) { tau[i] = INFINITY; cnt[i] = 0; }
    if (i < 2) ccount[i] = 0;
}

// ---- the distance tiles
// Candidates only have to be found, not ranked (knn_rerank does that in double), so the dot
// products run on the bf16 matrix cores at sixteen times the rate of the fp32 ones: every value
// is split as x = hi + lo + rest, hi = bf16(x), lo = bf16(x - hi), |rest| <= 2^-18 |x|, and
// q.x is taken as sum hi.hi + hi.lo + lo.hi, accumulated in fp32.  What this leaves out, and
// what the accumulation rounds away, is bounded in tile_error_coeff(); knn_rerank certifies
// each row against that bound, so the neighbour lists stay exact.
//
// split_bf16 lays the two parts out for the tile kernel: row-major, the row padded to a multiple
// of SLAB columns, and per SLAB columns the 32 high parts followed by the 32 low parts (128 bytes,
// the piece of a row that one LDS slab holds).
constexpr int SLAB = 32;                  // columns per LDS slab (two matrix-core steps of 16)
constexpr int SLAB_ROW = 4 * SLAB;        // bytes of a row's piece of a slab
constexpr int LDS_ROW = SLAB_ROW + 16;    // padded: 8 consecutive rows' 16-byte reads hit distinct banks

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__global__ __launch_bounds__(256) void split_bf16(const float *__restrict__ X, const float *__restrict__ mu, int n, int d,
                                                  int dp, const int *__restrict__ rowmap, int nsrc,
                                                  uint16_t *__restrict__ Xs)
{
    const size_t e = global_index();
    if (e >= (size_t)n * dp) return;
    const size_t row = e / dp;
    const int k = (int)(e % dp);
    const size_t src = rowmap ? (size_t)min(max(rowmap[row], 0), nsrc - 1) : row;
    const float x = k < d ? X[src * d + k] - mu[k] : 0.f;
    const uint32_t hi = bf16_rne(x);
    const uint32_t lo = bf16_rne(x - __uint_as_float(hi << 16));      // the difference is exact in fp32
    uint16_t *o = Xs + row * dp * 2 + (size_t)(k / SLAB) * (2 * SLAB) + (k % SLAB);
    o[0] = (uint16_t)hi;
    o[SLAB] = (uint16_t)lo;
}

// The values in half precision, for the first sweep over long rows: row-major, rows padded to a multiple of 64
// columns, scaled by a power of two (`scale`) that brings the largest magnitude just below 2^15: nothing overflows,
// and what is too small for a normal half is below 2^-28 of the largest magnitude.
__global__ __launch_bounds__(256) void split_high(const float *__restrict__ X, const float *__restrict__ mu, int n, int d,
                                                  int dph, float scale, uint16_t *__restrict__ Xh)
{
    const size_t e = global_index();
    if (e >= (size_t)n * dph) return;
    const size_t row = e / dph;
    const int k = (int)(e % dph);
    const _Float16 h = (_Float16)(k < d ? (X[row * d + k] - mu[k]) * scale : 0.f);     // round to nearest even
    Xh[e] = __builtin_bit_cast(uint16_t, h);
}

// max |x - mu| over all values, as the bits of a non-negative float (they order like the values)
__global__ __launch_bounds__(256) void max_abs_centred(const float *__restrict__ X, const float *__restrict__ mu, size_t total,
                                                       int d, unsigned int *__restrict__ out)
{
    float v = 0.f;
    for (size_t i = global_index(); i < total; i += (size_t)gridDim.x * gridDim.y * blockDim.x)
        v = fmaxf(v, fabsf(X[i] - mu[i % d]));
    v = wave_max(v);
    if (lane_id() == 0) atomicMax(out, __float_as_uint(v));
}

// Bound on |computed - exact| of one tile distance, as a multiple of |q|^2 + |x|^2.
//   split: the products left out (lo.lo, rest.x, x.rest) are at most 3 (1 + 2^-18) 2^-18 |q_t x_t| each;
//   accumulation: a sum reaches the result through at most R fp32 additions, R = 3 * (columns per
//     flush) + number of flushes; each is taken to lose up to 2^-23 relative (one unit in the last
//     place, which also covers truncating adders), so the sum is off by R 2^-23 / (1 - R 2^-23)
//     times the sum of |terms| <= (1 + 2^-8)^2 sum |q_t x_t|;
//   sum |q_t x_t| <= (|q|^2 + |x|^2) / 2, and the distance takes -2 times the dot product;
//   norms (each a rounded double sum), their sum and the final fused multiply-add: 8 more roundings
//   of quantities below 2 (|q|^2 + |x|^2);
//   centring: q' = fl(q - mu), x' = fl(x - mu) are off by 2^-24 relative per coordinate, which moves
//   |q' - x'|^2 by at most 2 |q - x| 2^-24 (|q'| + |x'|) <= 4 2^-24 (|q'|^2 + |x'|^2) (and a second-order term).
// 5 % on top for the norms themselves being rounded values.  q, x here are the centred rows.
// high_only: the tiles multiply the values rounded to half precision (one product per coordinate): what is left
// out is then q ex + eq x - eq ex with |eq| <= 2^-11 |q|, |ex| <= 2^-11 |x|, at most (2^-10 + 2^-22) |q_t x_t|
// (values too small for a normal half are covered by an additive term, see high_first_extra()).
__host__ __device__ inline double tile_error_coeff(int d, bool two_level, bool high_only = false)
{
    const int dp = (d + SLAB - 1) / SLAB * SLAB;
    const double per = high_only ? 1.0 : 3.0;      // products per coordinate
    const double R = two_level ? per * KFLUSH + (double)((dp + KFLUSH - 1) / KFLUSH) : per * dp;
    const double u = 1.1920928955078125e-07;   // 2^-23
    const double split = high_only ? 0.0009765625 + 2.384185791015625e-07
                                   : 3.0 * (1.0 + 3.814697265625e-06) * 3.814697265625e-06;
    const double accum = 1.0079 * R * u / (1.0 - R * u);
    return 1.05 * (split + accum + (16.0 + 4.2) * 5.9604644775390625e-08);
}

// A wave's queue of accepted pairs lives in LDS.
typedef __attribute__((address_space(3))) uint64_t lds_u64;
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(3))) float lds_f32;

// A wave appends the `fill` pairs it has queued to their rows' candidate buffers.
__device__ __forceinline__ void append_queue_inline(const lds_u32 *qrow, const lds_u64 *qkey, int fill, int *__restrict__ cnt,
                                                    uint64_t *__restrict__ cand, int cap)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int e = (int)lane_id(); e < fill; e += WAVE) {
        const uint32_t row = qrow[e];
        const int pos = atomicAdd(&cnt[row], 1);
        if (pos < cap) cand[(size_t)row * cap + pos] = qkey[e];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __noinline__ void append_queue(const lds_u32 *qrow, const lds_u64 *qkey, int fill, int *__restrict__ cnt,
                                          uint64_t *__restrict__ cand, int cap)
{
    append_queue_inline(qrow, qkey, fill, cnt, cand, cap);
}

// The rare path of a tile's epilogue (some lane of the wave found a pair under its row's cut-off),
// out of line so that the unrolled test loop stays a handful of instructions per pair.  Called
// with all lanes active; queues the pairs (slots from a ballot) and returns the new fill level.
// ql: the lane's query row within the tile (row qa + ql of X, row qa + ql - q0 of the block).
// A leaf on purpose: a function that calls another one saves its return address through memory.
// qid (or null): the tile's query rows are not consecutive; qid[ql] is the row of the lane's query.
__device__ __noinline__ int queue_pairs(bool near, int j, int ql, int qa, int q0, const lds_f32 *qn, float nj, float dot,
                                        int fill, int qcap, lds_u64 *qkey, lds_u32 *qrow, int *__restrict__ cnt,
                                        uint64_t *__restrict__ cand, int cap, const lds_u32 *qid, int exclude_self,
                                        const int *__restrict__ selfmap)
{
    const int q = qid ? (int)qid[ql] : qa + ql;
    // (selfmap: query q is row selfmap[q] of the database)
    const bool take = near && (!exclude_self || j != (selfmap ? selfmap[q] : q));
    const uint64_t m = __ballot(take);
    if (m == 0) return fill;
    if (fill + WAVE > qcap) { append_queue_inline(qrow, qkey, fill, cnt, cand, cap); fill = 0; }
    if (take) {
        const int slot = fill + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        const float dist = (qn[ql] + nj) - 2.0f * dot;
        qkey[slot] = ((uint64_t)orderable(dist) << 32) | (uint32_t)j;
        qrow[slot] = (uint32_t)(q - q0);
    }
    return fill + __popcll(m);
}

// MB x 2 blocks of 32 x 32 per wave, 2 x 2 waves: 64 MB query rows [q0 + 64 MB bx, ..) against 128
// database rows [j0 + 128 by, ..).  MB = 4 (256 x 128) halves the bytes loaded per product, which
// is what bounds the kernel once the matrix cores run at the bf16 rate.
// TWO: two-level accumulation, needed once d exceeds KFLUSH: the matrix cores sum KFLUSH columns
// into `part`, which is then added to `acc` and cleared, so the accumulation error stays that of
// a short sum.  It doubles the accumulator registers, hence MB = 2 there.
// Xb, norms_b: the database rows and their norms (Xs and norms again when the rows are searched among themselves,
// exclude_self = 1: a row is not its own neighbour).
// GATHER: the tiles of an inverted-file search (Eq. (11)) instead of a rectangle of the all-pairs matrix.  The
// rows are in list order (cellptr[L] .. cellptr[L+1] hold list L); the queries of the pass that probe list L at
// the current rank are pairq[pairptr[L] .. pairptr[L+1]) (row numbers, any order); a launch takes the rows
// chunk * DBC .. of every list.  Workgroup t < tptr[nlist] belongs to the list L with tptr[L] <= t < tptr[L+1] and
// is tile (a, b) of its ceil(queries / TQ) x ceil(rows of the chunk / TN) tiles; workgroups past the end leave.
template <int MB, bool TWO, bool GATHER>
__global__ __launch_bounds__(256, 2) void knn_tile_mfma(const uint4 *__restrict__ Xs, int dp, int q0, int qend, int j0,
                                                        int jend, const float *__restrict__ norms,
                                                        const float *__restrict__ tau, int *__restrict__ cnt,
                                                        uint64_t *__restrict__ cand, int cap, int *__restrict__ ccount,
                                                        const uint4 *__restrict__ Xb, const float *__restrict__ norms_b,
                                                        int exclude_self, const int *__restrict__ selfmap,
                                                        const int *__restrict__ tptr, int nlist,
                                                        const int *__restrict__ pairptr, const int *__restrict__ pairq,
                                                        const int *__restrict__ cellptr, int chunk)
{
    static_assert(!TWO || MB == 2, "two-level accumulation has registers for 2 x 2 blocks only");
    constexpr int TQ = 64 * MB;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *ccount = 0;   // for the compaction pass that follows
    __shared__ __align__(16) unsigned char As[TQ * LDS_ROW];
    __shared__ __align__(16) unsigned char Bs[TN * LDS_ROW];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    int qa = q0 + blockIdx.x * TQ, ja = j0 + blockIdx.y * TN;
    int po = 0, nq = TQ;            // GATHER: first entry of pairq and number of queries of this tile
    if (GATHER) {
        const int t = (int)blockIdx.x;
        if (t >= tptr[nlist]) return;
        int lo = 0, hi = nlist;     // tptr[lo] <= t < tptr[hi]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (tptr[mid] <= t) lo = mid; else hi = mid;
        }
        const int nql = pairptr[lo + 1] - pairptr[lo];
        const int rs = min(cellptr[lo] + chunk * DBC, cellptr[lo + 1]), re = min(cellptr[lo + 1], rs + DBC);
        const int tr = max((re - rs + TN - 1) / TN, 1);
        const int a = (t - tptr[lo]) / tr, b = (t - tptr[lo]) % tr;
        po = pairptr[lo] + a * TQ;
        nq = max(min(TQ, nql - a * TQ), 0);
        ja = rs + b * TN;
        jend = min(re, ja + TN);
        qa = 0;
    }
    const int row16 = dp / 4;              // 16-byte pieces per row of Xs
    const int piece = tid & 7, lrow = tid >> 3;
    floatx16 acc[TWO ? MB : 1][TWO ? 2 : 1], part[MB][2];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (TWO) acc[TWO ? a : 0][TWO ? b : 0][i] = 0.f;
                part[a][b][i] = 0.f;
            }
    uint4 ra[2 * MB], rb[4];
    int arow[2 * MB];               // the query rows this thread loads (-1: none)
#pragma unroll
    for (int it = 0; it < 2 * MB; ++it) {
        const int lr = lrow + 32 * it;
        if (GATHER) arow[it] = lr < nq ? max(pairq[po + lr], 0) : -1;
        else arow[it] = qa + lr < qend ? qa + lr : -1;
    }
    auto load = [&](int slab) {
#pragma unroll
        for (int it = 0; it < 2 * MB; ++it)
            ra[it] = arow[it] >= 0 ? Xs[(size_t)arow[it] * row16 + slab * 8 + piece] : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = ja + lrow + 32 * it;
            rb[it] = r < jend ? Xb[(size_t)r * row16 + slab * 8 + piece] : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    load(0);
    const int r32 = lane & 31, h = lane >> 5;
    const int nslab = dp / SLAB;
    for (int slab = 0; slab < nslab; ++slab) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < 2 * MB; ++it)
            *reinterpret_cast<uint4 *>(As + (lrow + 32 * it) * LDS_ROW + piece * 16) = ra[it];
#pragma unroll
        for (int it = 0; it < 4; ++it)
            *reinterpret_cast<uint4 *>(Bs + (lrow + 32 * it) * LDS_ROW + piece * 16) = rb[it];
        __syncthreads();
        if (slab + 1 < nslab) load(slab + 1);
        // a lane holds 8 consecutive columns of its row for each step of 16: columns 8 h .. 8 h + 7.
        // Both operands use the same assignment, so the products pair up whatever order the
        // hardware sums them in.
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            // low.high, high.high, high.low, in that order so that at most three fragment sets are live
            bf16x8 ah[MB], al[MB], bh[2], bl[2];
            const unsigned char *pa = As + (wm * 32 * MB + r32) * LDS_ROW + ks * 32 + h * 16;
            const unsigned char *pb = Bs + (wn * 64 + r32) * LDS_ROW + ks * 32 + h * 16;
#pragma unroll
            for (int a = 0; a < MB; ++a)
                al[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pa + a * 32 * LDS_ROW + 2 * SLAB));
#pragma unroll
            for (int b = 0; b < 2; ++b)
                bh[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pb + b * 32 * LDS_ROW));
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    part[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[a], bh[b], part[a][b], 0, 0, 0);
#pragma unroll
            for (int a = 0; a < MB; ++a)
                ah[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pa + a * 32 * LDS_ROW));
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    part[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[a], bh[b], part[a][b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < 2; ++b)
                bl[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pb + b * 32 * LDS_ROW + 2 * SLAB));
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    part[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[a], bl[b], part[a][b], 0, 0, 0);
        }
        if (TWO && ((slab % (KFLUSH / SLAB)) == (KFLUSH / SLAB) - 1 || slab + 1 == nslab)) {
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        acc[TWO ? a : 0][TWO ? b : 0][i] += part[a][b][i];
                        part[a][b][i] = 0.f;
                    }
        }
    }
    // epilogue: lane holds column (lane % 32) and rows 8 (i / 4) + 4 (lane / 32) + i % 4 of each block.
    // The tile's query norms and cut-offs are staged once in LDS (the slabs are no longer needed).
    // Accepted pairs are few (well under 1 % once the cut-offs have settled), but nearly every wave
    // has some, and an append to a row's buffer is a returning atomic: done where the pair is found,
    // each would stall the wave for a round trip to memory.  So the wave first collects its pairs in
    // an LDS queue (slots from a ballot, no atomics) and appends them all at once, 64 at a time.
    // The test itself is |x|^2 - 2 q.x < cut-off - |q|^2 (one fused multiply-add and one compare per
    // pair); the distance as stored, (|q|^2 + |x|^2) - 2 q.x, is formed for accepted pairs only.
    // Both are within tile_error_coeff() of the exact distance.
    __syncthreads();
    float *qn = reinterpret_cast<float *>(As), *qd = qn + TQ;
    uint32_t *qid = reinterpret_cast<uint32_t *>(qd + TQ);
    for (int t = tid; t < TQ; t += 256) {
        const int q = GATHER ? (t < nq ? max(pairq[po + t], q0) : -1) : (qa + t < qend ? qa + t : -1);
        const float nrm = q >= 0 ? norms[q] : 0.f;
        qn[t] = nrm;
        qd[t] = q >= 0 ? tau[q - q0] - nrm : -INFINITY;     // rows past the end accept nothing
        if (GATHER) qid[t] = (uint32_t)max(q, 0);
    }
    __syncthreads();
    constexpr int QCAP = 320;
    static_assert(4 * QCAP * 12 <= TN * LDS_ROW, "the queues live where the database slab was");
    lds_u64 *qkey = (lds_u64 *)(Bs) + w * QCAP;
    lds_u32 *qrow = (lds_u32 *)(Bs + 4 * QCAP * 8) + w * QCAP;
    int fill = 0;       // wave-uniform
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int j = ja + wn * 64 + b * 32 + r32;
        const float nj = j < jend ? norms_b[j] : INFINITY;    // rows past the end are never closer than any cut-off
#pragma unroll
        for (int a = 0; a < MB; ++a) {
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int ql0 = wm * 32 * MB + a * 32 + 8 * i4 + 4 * h;
                const float4 d4 = *reinterpret_cast<const float4 *>(qd + ql0);
                const float dq[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    const int i = 4 * i4 + ii;
                    const float dot = TWO ? acc[TWO ? a : 0][TWO ? b : 0][i] : part[a][b][i];
                    const bool near = fmaf(-2.0f, dot, nj) < dq[ii];
                    if (__ballot(near) != 0)
                        fill = __builtin_amdgcn_readfirstlane(queue_pairs(near, j, ql0 + ii, qa, q0, (const lds_f32 *)qn, nj, dot, fill, QCAP,
                                                                          qkey, qrow, cnt, cand, cap,
                                                                          GATHER ? (const lds_u32 *)qid : (const lds_u32 *)nullptr,
                                                                          exclude_self, selfmap));
                }
            }
        }
    }
    append_queue(qrow, qkey, fill, cnt, cand, cap);
}

// 16-byte piece c of an unpadded 128-byte LDS row r sits at position c ^ swz(r): see knn_tile_resident below
__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ ((row & 1) << 2)) & 7; }

// ---- the first sweep over long rows: half precision, 256 x 256 tiles
// One product per coordinate makes the operands, not the matrix work, the cost: with 256 x 128 tiles two workgroups
// per compute unit pull 10 TB/s out of the second-level cache.  A 256 x 256 tile needs a third less per product.  One
// workgroup of eight waves per compute unit (a wave owns 128 x 64 outputs, eight 32 x 32 blocks), and the overlap that
// several workgroups would give comes from the kernel itself.  The slabs of 64 columns alternate between two LDS
// buffers, which the loads fill directly (global_load_lds: no registers hold a slab in flight, and no LDS store
// instructions are issued); a wave's instruction brings eight rows of 128 bytes, unpadded, every lane taking the piece
// that the swizzle puts at its position.  There is one barrier per slab, in front of its last step: by then every wave
// has read all it needs of the current buffer, so the loads of the slab after the next go out right behind the barrier
// and have a whole slab's time to arrive, and the first fragments of the next slab are requested while the last
// products of this one run.  Within a step the next step's six fragment reads are placed by hand, one behind each
// of the first six products.  Rows as split_high leaves them (128 bytes per 64 columns); dot_scale undoes their scaling.
constexpr int HT = 256;                                 // tile: query rows = database rows
constexpr int HALF_THREADS = 512;
constexpr int HALF_BUF = 2 * HT * 128;                  // one buffer: the tile's query rows, then its database rows
constexpr size_t HALF_TILE_LDS = 2 * (size_t)HALF_BUF;

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

__global__ __launch_bounds__(HALF_THREADS, 1) void knn_tile_half(const uint4 *__restrict__ Xh, int dph, int q0, int qend, int j0,
                                                                 int jend, const float *__restrict__ norms,
                                                                 const float *__restrict__ tau, int *__restrict__ cnt,
                                                                 uint64_t *__restrict__ cand, int cap, int *__restrict__ ccount,
                                                                 float dot_scale)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *ccount = 0;   // for the compaction pass that follows
    extern __shared__ __align__(16) unsigned char hsm[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 2, wn = w & 3;
    // Workgroups go to the eight XCDs in turn, and each XCD has a second-level cache of its own.  Workgroup number
    // 8 l + x is XCD x's l-th: XCD x takes a strip of the query tiles and walks it query tile by query tile, all
    // database tiles of one query tile next to each other, so that the 32 workgroups an XCD runs at a time are a few
    // query tiles against all database tiles of the launch and find each other's rows in that cache (taken in plain
    // row-major order, every tile's rows came from memory: 3-4 TB/s of re-reads, which is what bounded the kernel).
    const int nqt = (qend - q0 + HT - 1) / HT, njt = (jend - j0 + HT - 1) / HT, per = (nqt + 7) / 8;
    const int xcd = (int)(blockIdx.x & 7u), local = (int)(blockIdx.x >> 3);
    const int qt = xcd * per + local / njt, jt = local % njt;
    if (qt >= nqt || local / njt >= per) return;       // (the grid is 8 per njt workgroups; the same for all lanes)
    const int qa = q0 + qt * HT, ja = j0 + jt * HT;
    const int row16 = dph / 8;              // 16-byte pieces per row
    const int r32 = lane & 31, h = lane >> 5;
    const int nslab = dph / (2 * SLAB);
    floatx16 acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
    // What this lane loads: wave w brings rows 32 w .. 32 w + 31 of both operands, eight rows an instruction; the
    // lane's row is 8 it + lane / 8 of them and its LDS position lane % 8, so it reads piece (lane % 8) ^ swz(row).
    // A row past the end is read as the last row: its products are finite and the epilogue accepts nothing for it.
    const uint4 *ga[4], *gb[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int lr = 32 * w + 8 * it + (lane >> 3), c = (lane & 7) ^ swz(lr);
        ga[it] = Xh + (size_t)min(qa + lr, qend - 1) * row16 + c;
        gb[it] = Xh + (size_t)min(ja + lr, jend - 1) * row16 + c;
    }
#define HALF_LOAD(slab_, buf_)                                                             \
    _Pragma("unroll") for (int it = 0; it < 4; ++it) {                                     \
        unsigned char *d_ = hsm + (size_t)(buf_) * HALF_BUF + (32 * w + 8 * it) * 128;     \
        __builtin_amdgcn_global_load_lds((glb_void *)(ga[it] + (size_t)(slab_) * 8), (lds_void *)d_, 16, 0, 0);              \
        __builtin_amdgcn_global_load_lds((glb_void *)(gb[it] + (size_t)(slab_) * 8), (lds_void *)(d_ + HT * 128), 16, 0, 0); \
    }
    // fragments: lane (r32, h) of block a reads piece 2 ks + h of row 32 a + r32 (swz depends on r32 alone)
    const int sw = swz(r32);
    const int fa_off = (wm * 128 + r32) * 128, fb_off = (HT + wn * 64 + r32) * 128;
    int pk[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) pk[ks] = ((2 * ks + h) ^ sw) * 16;
    halfx8 fa[2][4], fb[2][2];
#define HALF_FRAGS(buf_, ks_, set_)                                                        \
    {                                                                                      \
        const unsigned char *b_ = hsm + (size_t)(buf_) * HALF_BUF + pk[ks_];               \
        _Pragma("unroll") for (int a = 0; a < 4; ++a)                                      \
            fa[set_][a] = __builtin_bit_cast(halfx8, *reinterpret_cast<const uint4 *>(b_ + fa_off + a * 32 * 128)); \
        _Pragma("unroll") for (int b = 0; b < 2; ++b)                                      \
            fb[set_][b] = __builtin_bit_cast(halfx8, *reinterpret_cast<const uint4 *>(b_ + fb_off + b * 32 * 128)); \
    }
#define HALF_PRODUCTS(set_)                                                                \
    _Pragma("unroll") for (int a = 0; a < 4; ++a)                                          \
        _Pragma("unroll") for (int b = 0; b < 2; ++b)                                      \
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[set_][a], fb[set_][b], acc[a][b], 0, 0, 0);
#define HALF_INTERLEAVE()                                                                  \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);         /* one matrix product */     \
    _Pragma("unroll") for (int i_ = 0; i_ < 6; ++i_) {                                     \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     /* one LDS read */           \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                 \
    }                                                                                      \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    HALF_LOAD(0, 0)
    if (nslab > 1) HALF_LOAD(1, 1)
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");     // (the first slab; all of them if there is only one)
    if (nslab == 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    HALF_FRAGS(0, 0, 0)
    for (int slab = 0; slab < nslab; ++slab) {
        const int cur = slab & 1, oth = cur ^ 1;
        HALF_FRAGS(cur, 1, 1)
        HALF_PRODUCTS(0)
        HALF_INTERLEAVE()
        __builtin_amdgcn_sched_barrier(0);
        HALF_FRAGS(cur, 2, 0)
        HALF_PRODUCTS(1)
        HALF_INTERLEAVE()
        __builtin_amdgcn_sched_barrier(0);
        HALF_FRAGS(cur, 3, 1)
        HALF_PRODUCTS(0)
        HALF_INTERLEAVE()
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this wave's part of the next slab has arrived
        __syncthreads();        // the other buffer is complete; nobody reads this one any more
        __builtin_amdgcn_sched_barrier(0);
        if (slab + 2 < nslab) HALF_LOAD(slab + 2, cur)
        // (past the last slab these fragments are read from a buffer nobody fills any more, and never used)
        HALF_FRAGS(oth, 0, 0)
        HALF_PRODUCTS(1)
        HALF_INTERLEAVE()
        __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();            // (the epilogue reuses the buffers)
#undef HALF_LOAD
#undef HALF_FRAGS
#undef HALF_PRODUCTS
#undef HALF_INTERLEAVE
    // epilogue, as in knn_tile_mfma: lane holds column (lane % 32) and rows 8 (i / 4) + 4 (lane / 32) + i % 4 of each
    // block; norms and cut-offs of the tile's queries staged in LDS, accepted pairs queued per wave
    float *qn = reinterpret_cast<float *>(hsm), *qd = qn + HT;
    for (int t = tid; t < HT; t += HALF_THREADS) {
        const int q = qa + t < qend ? qa + t : -1;
        const float nrm = q >= 0 ? norms[q] : 0.f;
        qn[t] = nrm;
        qd[t] = q >= 0 ? tau[q - q0] - nrm : -INFINITY;     // rows past the end accept nothing
    }
    __syncthreads();
    constexpr int QCAP = 320;
    unsigned char *qbase = hsm + 4096;
    lds_u64 *qkey = (lds_u64 *)(qbase) + w * QCAP;
    lds_u32 *qrow = (lds_u32 *)(qbase + 8 * QCAP * 8) + w * QCAP;
    int fill = 0;       // wave-uniform
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int j = ja + wn * 64 + b * 32 + r32;
        const float nj = j < jend ? norms[j] : INFINITY;    // rows past the end are never closer than any cut-off
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int ql0 = wm * 128 + a * 32 + 8 * i4 + 4 * h;
                const float4 d4 = *reinterpret_cast<const float4 *>(qd + ql0);
                const float dq[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    const float dot = acc[a][b][4 * i4 + ii] * dot_scale;
                    const bool near = fmaf(-2.0f, dot, nj) < dq[ii];
                    if (__ballot(near) != 0)
                        fill = __builtin_amdgcn_readfirstlane(queue_pairs(near, j, ql0 + ii, qa, q0, (const lds_f32 *)qn, nj, dot, fill, QCAP,
                                                                          qkey, qrow, cnt, cand, cap, (const lds_u32 *)nullptr, 1,
                                                                          (const int *)nullptr));
                }
            }
        }
    }
    append_queue(qrow, qkey, fill, cnt, cand, cap);
}

// ---- d <= 64: the query tile stays in LDS
// With two slabs at most, the kernel above spends its time waiting: a workgroup makes five
// dependent round trips to memory (two slabs, norms and cut-offs, the appends) around 2 x 48 matrix
// instructions.  Here a workgroup keeps its 256 query rows on chip for the whole launch (each
// wave holds the fragments of its 64 rows in registers) and walks over the database rows; the
// next rows are in flight (registers) while the current ones are multiplied and tested.  The
// workgroup is the only one that appends to its rows' buffers during the launch, so the fill
// counts live in LDS: an append is an LDS atomic and a store that nobody waits for.
// Eight waves in two groups of four: each group takes every other tile of 128 database rows, in
// two halves of 64; a wave holds 64 x 64 of its group's 256 x 64 products.  Group 0 multiplies a
// half and then tests it, group 1 tests its previous half first and then multiplies the next, so
// that on every SIMD one wave feeds the matrix cores while the other one runs the tests on the
// vector unit.  (Two halves per trip: one half's work is shorter than a load takes to arrive.)
// LDS rows are 128 bytes (32 high parts, 32 low parts), unpadded; the 16-byte piece c of row r sits
// at position c ^ swz(r), chosen so that 16 consecutive rows' reads of one piece fall on 16
// different 16-byte bank groups of a 256-byte LDS line (and 8 consecutive rows on 8 of a
// 128-byte line), while the 8 pieces of a row stay a permutation of the row.
constexpr int RQ = 256;          // query rows per workgroup
constexpr int RT = 128;          // database rows per group and trip, taken in two halves
constexpr int RESIDENT_MIN_ROWS = 64 * RQ;   // fewer query rows than this leave most compute units without a workgroup

constexpr size_t resident_lds_bytes(int ns)
{
    return 2 * (size_t)ns * RT * SLAB_ROW + 3 * RQ * 4;
}


// A workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// store of the wave to complete, which would put the appends' trip to memory on the critical path.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int NS>
__global__ __launch_bounds__(512, 1) void knn_tile_resident(const uint4 *__restrict__ Xs, int q0, int qend, int j0, int jend,
                                                            const float *__restrict__ norms,
                                                            const float *__restrict__ tau, int *__restrict__ cnt,
                                                            uint64_t *__restrict__ cand, int cap, int kp, int force,
                                                            int *__restrict__ clist, int *__restrict__ ccount,
                                                            int *__restrict__ ccount_next)
{
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *Bs = smem;                                   // [2 groups][NS][RT] rows
    float *qn = reinterpret_cast<float *>(Bs + 2 * NS * RT * SLAB_ROW), *qd = qn + RQ;
    int *qc = reinterpret_cast<int *>(qd + RQ);                 // candidates in each row's buffer
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int g = w >> 2, wq = w & 3;
    const int r32 = lane & 31, h = lane >> 5, sw = swz(r32);
    const int qa = q0 + blockIdx.x * RQ;
    constexpr int row16 = NS * 8;          // 16-byte pieces per row of Xs
    if (blockIdx.x == 0 && tid == 0) *ccount_next = 0;   // the list of the next launch (nobody reads it any more)
    // the wave's query fragments: [block][slab][step] high and low parts, as the matrix cores take them
    bf16x8 afh[2][NS][2], afl[2][NS][2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int r = qa + wq * 64 + a * 32 + r32;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const uint4 z = make_uint4(0u, 0u, 0u, 0u);
                afh[a][sl][ks] = __builtin_bit_cast(bf16x8, r < qend ? Xs[(size_t)r * row16 + sl * 8 + 2 * ks + h] : z);
                afl[a][sl][ks] = __builtin_bit_cast(bf16x8, r < qend ? Xs[(size_t)r * row16 + sl * 8 + 4 + 2 * ks + h] : z);
            }
    }
    for (int t = tid; t < RQ; t += 512) {
        const int q = qa + t;
        const float nq = q < qend ? norms[q] : 0.f;
        qn[t] = nq;
        qd[t] = q < qend ? tau[q - q0] - nq : -INFINITY;     // rows past the end accept nothing
        qc[t] = q < qend ? cnt[q - q0] : 0;
    }
    unsigned char *Bg = Bs + g * NS * RT * SLAB_ROW;
    const int bpiece = tid & 7, blrow = (tid & 255) >> 3;
    const int ntile = (jend - j0 + RT - 1) / RT, npair = (ntile + 1) / 2;
    uint4 rb[4 * NS];
    float njn[2][2];   // |x|^2 of this lane's two columns of each half of the tile in rb
    auto load_tile = [&](int pair) {
        const int ja = j0 + (2 * pair + g) * RT;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int r = ja + blrow + 32 * it;
#pragma unroll
            for (int sl = 0; sl < NS; ++sl)
                rb[it * NS + sl] = r < jend ? Xs[(size_t)r * row16 + sl * 8 + bpiece] : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int j = ja + hf * 64 + b * 32 + r32;
                njn[hf][b] = j < jend ? norms[j] : INFINITY;    // rows past the end are never closer than any cut-off
            }
    };
    floatx16 part[2][2];
    float njc[2] = {INFINITY, INFINITY};   // the same for the half in `part`
    int jac = j0;                          // first database row of that half
    auto test_tile = [&]() {
        // one base per lane, the rest compile-time offsets (and no addresses carried around the loop)
        int lbase = wq * 64 + 4 * h;
        asm volatile("" : "+v"(lbase));
        const float *qd_l = qd + lbase, *qn_l = qn + lbase;
        int *qc_l = qc + lbase;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int j = jac + b * 32 + r32;
            const float nj = njc[b];
#pragma unroll
            for (int a = 0; a < 2; ++a) {
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const float4 d4 = *reinterpret_cast<const float4 *>(qd_l + a * 32 + 8 * i4);
                    const float dq[4] = {d4.x, d4.y, d4.z, d4.w};
                    // four pairs per branch: a branch on a vector compare waits for the compare, and that
                    // wait, not the arithmetic, is what a test costs (sixteen per branch: slower again,
                    // the rare path is entered too often)
                    bool near[4];
#pragma unroll
                    for (int ii = 0; ii < 4; ++ii) near[ii] = fmaf(-2.0f, part[a][b][4 * i4 + ii], nj) < dq[ii];
                    if (__builtin_expect(__ballot(near[0] || near[1] || near[2] || near[3]) != 0, 0)) {
#pragma unroll
                        for (int ii = 0; ii < 4; ++ii) {
                            if (__ballot(near[ii]) == 0) continue;
                            const float dot = part[a][b][4 * i4 + ii];
                            const int off = a * 32 + 8 * i4 + ii;
                            const int q = qa + lbase + off;
                            if (near[ii] && j != q) {
                                const float dist = (qn_l[off] + nj) - 2.0f * dot;
                                const int pos = atomicAdd(qc_l + off, 1);
                                if (pos < cap)
                                    cand[(size_t)(q - q0) * cap + pos] = ((uint64_t)orderable(dist) << 32) | (uint32_t)j;
                            }
                        }
                    }
                }
            }
        }
    };
    if (npair > 0) load_tile(0);
    const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    bool have = false;      // group 1: `part` holds a half that has not been tested yet
    for (int pair = 0; pair < npair; ++pair) {
        lds_barrier();          // every wave is done with the tiles in LDS (first trip: the query rows are in)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = blrow + 32 * it;
#pragma unroll
            for (int sl = 0; sl < NS; ++sl)
                *reinterpret_cast<uint4 *>(Bg + (sl * RT + row) * SLAB_ROW + ((bpiece ^ swz(row)) << 4)) = rb[it * NS + sl];
        }
        const float njl[2][2] = {{njn[0][0], njn[0][1]}, {njn[1][0], njn[1][1]}};
        lds_barrier();
        // the next rows are requested after the first tests of this trip: a wait for them (the counter
        // is in order) then never covers stores made by tests, except those of the half in between
        for (int hf = 0; hf < 2; ++hf) {
            if (g == 1 && have) test_tile();
            if (hf == 0 && pair + 1 < npair) load_tile(pair + 1);
#pragma unroll
            for (int sl = 0; sl < NS; ++sl) {
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    // low.high, high.low, high.high; piece index = 4 (low part) + 2 ks + h
                    bf16x8 bh[2], bl[2];
                    const unsigned char *pb = Bg + (sl * RT + hf * 64 + r32) * SLAB_ROW;
                    const int ch = ((2 * ks + h) ^ sw) << 4, cl = ((4 + 2 * ks + h) ^ sw) << 4;
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        bh[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pb + b * 32 * SLAB_ROW + ch));
                        bl[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pb + b * 32 * SLAB_ROW + cl));
                    }
#pragma unroll
                    for (int a = 0; a < 2; ++a)
#pragma unroll
                        for (int b = 0; b < 2; ++b)
                            part[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afl[a][sl][ks], bh[b],
                                                                                 (sl == 0 && ks == 0) ? zero16 : part[a][b], 0, 0, 0);
#pragma unroll
                    for (int a = 0; a < 2; ++a)
#pragma unroll
                        for (int b = 0; b < 2; ++b)
                            part[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afh[a][sl][ks], bl[b], part[a][b], 0, 0, 0);
#pragma unroll
                    for (int a = 0; a < 2; ++a)
#pragma unroll
                        for (int b = 0; b < 2; ++b)
                            part[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afh[a][sl][ks], bh[b], part[a][b], 0, 0, 0);
                }
            }
            njc[0] = njl[hf][0];
            njc[1] = njl[hf][1];
            jac = j0 + (2 * pair + g) * RT + hf * 64;
            have = true;
            if (g == 0) test_tile();
        }
    }
    if (g == 1 && have) test_tile();
    lds_barrier();
    // the fill counts go back, and the rows whose buffers are due for compaction go on the list (the
    // rule of knn_compact_list, which this kernel makes unnecessary)
    for (int t = tid; t < RQ; t += 512) {
        const int q = qa + t;
        if (q < qend) {
            const int c = qc[t];
            cnt[q - q0] = c;
            const int cc = min(c, cap);
            if (cc >= kp && (force || !(qd[t] < INFINITY) || cc >= kp + COMPACT_SLACK || cc + COMPACT_EVERY * DBC > cap))
                clist[atomicAdd(ccount, 1)] = q - q0;    // any order
        }
    }
}

// Bitonic sort of `size` (power of two) 64-bit keys in LDS by a 256-thread block.
__device__ __forceinline__ void bitonic_sort(uint64_t *s, int size)
{
    for (int k = 2; k <= size; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < size; t += blockDim.x) {
                int ixj = t ^ j;
                if (ixj > t) {
                    uint64_t a = s[t], b = s[ixj];
                    bool up = (t & k) == 0;
                    if ((a > b) == up) { s[t] = b; s[ixj] = a; }
                }
            }
            __syncthreads();
        }
    }
}

// Which rows of the query block need their candidates compacted now (one thread per row; the
// compaction itself takes a workgroup per row, and on most slabs only a few rows need it).
__global__ __launch_bounds__(256) void knn_compact_list(const float *__restrict__ tau, const int *__restrict__ cnt,
                                                        int cap, int kp, int rows, int force, int *__restrict__ list,
                                                        int *__restrict__ count)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    int c = cnt[row];
    if (c > cap) c = cap;
    if (c < kp) return;                 // not yet k' candidates: the cut-off stays +inf
    // sort only when enough new candidates have piled up to matter, when the next slab could
    // overflow the buffer, or at the end (force); in between the cut-off is merely a bit stale
    if (!force && tau[row] < INFINITY && c < kp + COMPACT_SLACK && c + COMPACT_EVERY * DBC <= cap) return;
    list[atomicAdd(count, 1)] = row;    // any order
}

// One workgroup per listed row: keeps the best k' of the row's candidates, sorted, and lowers the
// cut-off to the k'-th.  The LDS buffer is sized for the usual case (k' and a few hundred new
// candidates), so that many rows are in flight per compute unit; a longer buffer (the first slabs
// of a query block) goes through it in several rounds, each keeping the best k' so far.
template <int BUF, int THREADS>
__global__ __launch_bounds__(THREADS) void knn_compact(float *__restrict__ tau, int *__restrict__ cnt,
                                                       uint64_t *__restrict__ cand, int cap, int kp, int rows,
                                                       const int *__restrict__ list, const int *__restrict__ count)
{
    __shared__ uint64_t s[BUF];
    const int m = min(*count, rows);
    for (int i = blockIdx.x; i < m; i += gridDim.x) {
        const int row = min(max(list[i], 0), rows - 1);
        int c = cnt[row];
        // (more pairs than the buffer holds cannot arrive between two passes as the launches are sized; should it
        // happen all the same, pairs were dropped: the cut-off goes to -inf for good, which fails the row's certificate)
        const bool lost = c > cap || tau[row] == -INFINITY;
        if (c > cap) c = cap;
        uint64_t *buf = cand + (size_t)row * cap;
        int done = 0, have = 0;         // candidates read so far; sorted survivors in s[0 .. have)
        while (done < c) {
            __syncthreads();            // the previous round (or row) is out of s
            const int take = min(BUF - have, c - done), total = have + take;
            int size = 1;
            while (size < total) size <<= 1;
            for (int t = threadIdx.x; t < size - have; t += THREADS) s[have + t] = t < take ? buf[done + t] : ~0ull;
            __syncthreads();
            bitonic_sort(s, size);
            done += take;
            have = min(total, kp);
        }
        for (int t = threadIdx.x; t < have; t += THREADS) buf[t] = s[t];
        if (threadIdx.x == 0 && have > 0) {
            cnt[row] = have;
            tau[row] = lost ? -INFINITY : have >= kp ? unorderable((uint32_t)(s[kp - 1] >> 32)) : tau[row];
        }
    }
}

// Exact distances of the candidates, final order, certificate.  One block per query.
// Query number i = q0 + block is row qmap[i] of X (row i if qmap is null); candidate number j is row cmap[j] of Y
// (row j); distances are taken from those rows, equal distances are ordered by the candidates' row numbers, which
// are also what is written, to row omap[i] (row i) of the result.  n_all: how many candidates a query can have at
// all (one that has them all needs no certificate).  norms_q by query number, norm_max over the database; coeff:
// tile_error_coeff() of the tiles that found the candidates, e_add: what else their distances may be off by.  A query without a certificate is listed as failmap[i] (i).
__global__ __launch_bounds__(256) void knn_rerank(const float *__restrict__ X, int nx, int d, const int *__restrict__ qmap,
                                                  const float *__restrict__ Y, int ny, const int *__restrict__ cmap,
                                                  const int *__restrict__ omap, const int *__restrict__ failmap, int q0,
                                                  int rows, int k, int kp, int n_all, double coeff, double e_add,
                                                  const float *__restrict__ norms_q, float norm_max,
                                                  const float *__restrict__ tau, const int *__restrict__ cnt,
                                                  const uint64_t *__restrict__ cand, int cap,
                                                  int32_t *__restrict__ knn_idx, double *__restrict__ knn_d2,
                                                  int *__restrict__ fail_count, int *__restrict__ fail_rows)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *xi = reinterpret_cast<float *>(smem);                       // d floats
    double *dd = reinterpret_cast<double *>(smem + up((size_t)d * 4)); // MAX_KP doubles
    __shared__ uint64_t key[MAX_KP];
    __shared__ int order[MAX_KP];
    __shared__ int cid[MAX_KP];          // the candidates' row numbers in Y
    const int row = blockIdx.x;
    if (row >= rows) return;
    const int i = q0 + row;
    int c = cnt[row];
    if (c > kp) c = kp;
    const int iu = min(max(qmap ? qmap[i] : i, 0), nx - 1);
    const float *x = X + (size_t)iu * d;
    for (int t = threadIdx.x; t < d; t += blockDim.x) xi[t] = x[t];
    const uint64_t *buf = cand + (size_t)row * cap;
    for (int a = threadIdx.x; a < c; a += blockDim.x) {
        const int j = (int)(uint32_t)buf[a];
        cid[a] = min(max(cmap ? cmap[min(j, ny - 1)] : j, 0), ny - 1);
    }
    __syncthreads();
    const int w = threadIdx.x >> 6;
    if (d % 4 == 0 && (reinterpret_cast<uintptr_t>(Y) & 15) == 0) {
        // rows of whole 16-byte pieces: a lane takes four coordinates a load and keeps four partial sums; a wave
        // has two candidates' rows in flight
        const float4 *x4 = reinterpret_cast<const float4 *>(xi);
        const int d4 = d / 4;
        for (int cidx = w; cidx < c; cidx += 8) {
            const bool two = cidx + 4 < c;
            const float4 *ya = reinterpret_cast<const float4 *>(Y + (size_t)cid[cidx] * d);
            const float4 *yb = reinterpret_cast<const float4 *>(Y + (size_t)cid[two ? cidx + 4 : cidx] * d);
            double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0, b0 = 0.0, b1 = 0.0, b2 = 0.0, b3 = 0.0;
#pragma unroll 2
            for (int t = lane_id(); t < d4; t += WAVE) {
                const float4 q = x4[t], u = ya[t], v = yb[t];
                double df;
                df = (double)q.x - (double)u.x; a0 += df * df;
                df = (double)q.y - (double)u.y; a1 += df * df;
                df = (double)q.z - (double)u.z; a2 += df * df;
                df = (double)q.w - (double)u.w; a3 += df * df;
                df = (double)q.x - (double)v.x; b0 += df * df;
                df = (double)q.y - (double)v.y; b1 += df * df;
                df = (double)q.z - (double)v.z; b2 += df * df;
                df = (double)q.w - (double)v.w; b3 += df * df;
            }
            const double sa = wave_sum((a0 + a1) + (a2 + a3)), sb = wave_sum((b0 + b1) + (b2 + b3));
            if (lane_id() == 0) {
                dd[cidx] = sa;
                if (two) dd[cidx + 4] = sb;
            }
        }
    } else {
        for (int cidx = w; cidx < c; cidx += 4) {
            const float *y = Y + (size_t)cid[cidx] * d;
            double s = 0.0;
            for (int t = lane_id(); t < d; t += WAVE) { double df = (double)xi[t] - (double)y[t]; s += df * df; }
            s = wave_sum(s);
            if (lane_id() == 0) dd[cidx] = s;
        }
    }
    __syncthreads();
    // rank by (distance, index): c <= 2048, plain counting rank is enough
    for (int a = threadIdx.x; a < c; a += blockDim.x) key[a] = orderable64(dd[a]);
    __syncthreads();
    for (int a = threadIdx.x; a < c; a += blockDim.x) {
        const uint64_t ka = key[a];
        const int ja = cid[a];
        int r = 0;
        for (int b = 0; b < c; ++b) {
            const uint64_t kb = key[b];
            r += (kb < ka) || (kb == ka && cid[b] < ja);
        }
        order[r] = a;
    }
    __syncthreads();
    const size_t orow = (size_t)(omap ? min(max(omap[i], 0), nx - 1) : i);
    for (int r = threadIdx.x; r < k && r < c; r += blockDim.x) {
        const int a = order[r];
        knn_idx[orow * k + r] = (int32_t)cid[a];
        if (knn_d2) knn_d2[orow * k + r] = dd[a];
    }
    if (threadIdx.x == 0) {
        // pairs never kept had single-precision distance >= tau; the error of that distance is
        // at most E, so they are farther than the exact k-th candidate if tau - E > D_k
        bool ok = c >= k;
        if (ok && c < n_all) {
            // (the additive term covers matrix cores that flush denormal bf16 parts to zero)
            const double E = coeff * ((double)norms_q[i] + (double)norm_max) + 1e-30 * d + e_add;
            const double Dk = dd[order[k - 1]];
            ok = (double)tau[row] - E > Dk;
        }
        if (!ok) fail_rows[atomicAdd(fail_count, 1)] = failmap ? failmap[i] : i;
    }
}

// ---- rows that failed the certificate: exact distances to every row, then selection
// A batch of `nb` failed rows rows[0..nb) at a time: okey[f * n + j] = ordered key of the exact distance
// between rows[f] and j.  A wave holds one database row in registers and meets every failed row
// (which come from the second-level cache), so X is read from memory once per batch.
constexpr int EXACT_MAX_D = 4096;
// (queries: rows qmap[rows[f]] of X, or rows[f]; database: the ny rows of Y; exclude_self: X and Y are the same rows)
__global__ __launch_bounds__(256) void knn_exact_dists(const float *__restrict__ X, int nx, const int *__restrict__ qmap,
                                                       const float *__restrict__ Y, int ny, int d,
                                                       const int *__restrict__ rows, int nb, int exclude_self,
                                                       uint64_t *__restrict__ okey)
{
    const size_t w = global_index() >> 6;
    if (w >= (size_t)ny) return;
    const int j = (int)w;
    const float *y = Y + (size_t)j * d;
    float yr[EXACT_MAX_D / WAVE];
#pragma unroll
    for (int q = 0; q < EXACT_MAX_D / WAVE; ++q) {
        const int t = q * WAVE + lane_id();
        yr[q] = (q * WAVE < d && t < d) ? y[t] : 0.f;
    }
    for (int f = 0; f < nb; ++f) {
        int i = rows[f];
        if (qmap) i = qmap[i];
        i = min(max(i, 0), nx - 1);
        const float *x = X + (size_t)i * d;
        double s = 0.0;
#pragma unroll
        for (int q = 0; q < EXACT_MAX_D / WAVE; ++q) {
            if (q * WAVE < d) {
                const int t = q * WAVE + lane_id();
                const double df = t < d ? (double)x[t] - (double)yr[q] : 0.0;
                s += df * df;
            }
        }
        s = wave_sum(s);
        if (lane_id() == 0) okey[(size_t)f * ny + j] = (exclude_self && j == i) ? ~0ull : orderable64(s);
    }
}

// One block: 8 radix passes over the ordered 64-bit keys find the k-th smallest distance; then
// the keys below it and the lowest-index ties are put in (distance, index) order.
constexpr int TIE_CAP = 4096;

__device__ __forceinline__ double key_to_double(uint64_t v)
{
    const uint64_t u = (v & 0x8000000000000000ull) ? (v & 0x7FFFFFFFFFFFFFFFull) : ~v;
    return __longlong_as_double((long long)u);
}

// One workgroup per failed row of the batch.  Row f of the batch has its keys at okey_all + f * stride: n of them,
// or counts[f] if counts is given; key j belongs to point j, or to point ids[f * stride + j] if ids is given
// (equal distances are ordered by that number); the list goes to row rows[f] of the output, or rowmap[rows[f]].
__global__ __launch_bounds__(1024) void knn_exact_select(const uint64_t *__restrict__ okey_all, size_t stride, int n,
                                                         const int *__restrict__ counts, const int *__restrict__ ids,
                                                         int k, const int *__restrict__ rows, const int *__restrict__ rowmap,
                                                         int nrows, int32_t *__restrict__ knn_idx, double *__restrict__ knn_d2)
{
    const uint64_t *okey = okey_all + (size_t)blockIdx.x * stride;
    const int *id = ids ? ids + (size_t)blockIdx.x * stride : nullptr;
    if (counts) n = min(counts[blockIdx.x], (int)stride);
    int i = min(max(rows[blockIdx.x], 0), nrows - 1);
    if (rowmap) i = min(max(rowmap[i], 0), nrows - 1);
    __shared__ uint32_t hist[256];
    __shared__ uint64_t prefix_s;
    __shared__ int want_s, nsel, ntie, best;
    __shared__ uint64_t selk[MAX_KP];
    __shared__ int selj[MAX_KP];
    __shared__ uint64_t tie[TIE_CAP];
    uint64_t prefix = 0;
    int want = k;   // rank (1-based) of the target among the keys that match the prefix so far
    for (int pass = 7; pass >= 0; --pass) {
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        const int sh = pass * 8;
        const uint64_t mask = pass == 7 ? 0ull : (~0ull << (sh + 8));
        for (int j = threadIdx.x; j < n; j += blockDim.x) {
            const uint64_t v = okey[j];
            if ((v & mask) == prefix) atomicAdd(&hist[(v >> sh) & 0xFF], 1u);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int acc = 0, b = 0;
            for (; b < 255; ++b) {
                if (acc + (int)hist[b] >= want) break;
                acc += (int)hist[b];
            }
            prefix_s = prefix | ((uint64_t)b << sh);
            want_s = want - acc;
        }
        __syncthreads();
        prefix = prefix_s;
        want = want_s;
        __syncthreads();
    }
    // prefix = k-th smallest key; k - want keys lie below it; `want` of its ties are needed
    if (threadIdx.x == 0) { nsel = 0; ntie = 0; }
    __syncthreads();
    for (int j = threadIdx.x; j < n; j += blockDim.x) {
        const uint64_t v = okey[j];
        if (v < prefix) {
            const int p = atomicAdd(&nsel, 1);
            if (p < MAX_KP) { selk[p] = v; selj[p] = id ? id[j] : j; }
        } else if (v == prefix) {
            const int p = atomicAdd(&ntie, 1);
            if (p < TIE_CAP) tie[p] = (uint64_t)(uint32_t)(id ? id[j] : j);
        }
    }
    __syncthreads();
    const int below = min(nsel, k - want);
    for (int a = threadIdx.x; a < below; a += blockDim.x) {
        const uint64_t ka = selk[a];
        const int ja = selj[a];
        int r = 0;
        for (int b = 0; b < below; ++b) r += (selk[b] < ka) || (selk[b] == ka && selj[b] < ja);
        knn_idx[(size_t)i * k + r] = ja;
        if (knn_d2) knn_d2[(size_t)i * k + r] = key_to_double(ka);
    }
    const double dk = key_to_double(prefix);
    if (ntie <= TIE_CAP) {
        int size = 1;
        while (size < ntie) size <<= 1;
        for (int t = threadIdx.x; t < size; t += blockDim.x) if (t >= ntie) tie[t] = ~0ull;
        __syncthreads();
        for (int kk = 2; kk <= size; kk <<= 1)
            for (int jj = kk >> 1; jj > 0; jj >>= 1) {
                for (int t = threadIdx.x; t < size; t += blockDim.x) {
                    const int ixj = t ^ jj;
                    if (ixj > t) {
                        const uint64_t a = tie[t], b = tie[ixj];
                        if ((a > b) == ((t & kk) == 0)) { tie[t] = b; tie[ixj] = a; }
                    }
                }
                __syncthreads();
            }
        for (int t = threadIdx.x; t < want && t < ntie; t += blockDim.x) {
            knn_idx[(size_t)i * k + below + t] = (int32_t)tie[t];
            if (knn_d2) knn_d2[(size_t)i * k + below + t] = dk;
        }
    } else {
        // more equidistant rows than the tie buffer holds: the lowest number above the last one taken, `want` times
        int last = -1;
        for (int out = below; out < k; ++out) {
            __syncthreads();
            if (threadIdx.x == 0) best = 0x7FFFFFFF;
            __syncthreads();
            int mine = 0x7FFFFFFF;
            for (int j = threadIdx.x; j < n; j += blockDim.x)
                if (okey[j] == prefix) {
                    const int v = id ? id[j] : j;
                    if (v > last && v < mine) mine = v;
                }
            if (mine != 0x7FFFFFFF) atomicMin(&best, mine);
            __syncthreads();
            last = best;
            if (last == 0x7FFFFFFF) break;
            if (threadIdx.x == 0) { knn_idx[(size_t)i * k + out] = last; if (knn_d2) knn_d2[(size_t)i * k + out] = dk; }
        }
    }
}

// ---- Eq. (1): conditional probabilities with the entropy fixed at ln(perplexity)
__device__ __forceinline__ double row_entropy(const double *__restrict__ dd, int k, double dmin, double beta)
{
    double S = 0.0, T = 0.0;
    for (int m = 0; m < k; ++m) {
        const double r = dd[m] - dmin;
        const double e = exp(-beta * r);
        S += e;
        T += r * e;
    }
    return log(S) + beta * T / S;
}

// One thread per row.  LDS: the workgroup's 64 rows of distances are staged in LDS (row stride k | 1
// doubles, so that the 64 threads' reads of their m-th distance fall in different banks) when they
// fit; the bisection re-reads them some forty times.
__global__ __launch_bounds__(64) void perplexity_search(const double *__restrict__ d2, int n, int k, double target,
                                                        double tol, double *__restrict__ cond,
                                                        int *__restrict__ unconverged, int staged)
{
    extern __shared__ __align__(16) unsigned char ps_smem[];
    double *sd = reinterpret_cast<double *>(ps_smem);
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int stride = k | 1;
    const double *dd = d2 + (size_t)min(i, n - 1) * k;
    if (staged) {
        const int row0 = blockIdx.x * 64, nrows = min(64, n - row0);
        const double *src = d2 + (size_t)row0 * k;
        for (int t = threadIdx.x; t < nrows * k; t += 64) sd[(t / k) * stride + t % k] = src[t];
        __syncthreads();
        dd = sd + threadIdx.x * stride;
    }
    if (i >= n) return;
    double dmin = dd[0];
    for (int m = 1; m < k; ++m) dmin = fmin(dmin, dd[m]);
    double lo = 0.0, hi = INFINITY, beta = 1.0;
    bool ok = false;
    for (int it = 0; it < 400; ++it) {
        const double H = row_entropy(dd, k, dmin, beta);
        if (fabs(H - target) <= tol) { ok = true; break; }
        if (H > target) { lo = beta; beta = isinf(hi) ? beta * 2.0 : 0.5 * (lo + hi); }
        else { hi = beta; beta = 0.5 * (lo + hi); }
        if (!(beta > 0.0) || isinf(beta)) break;
    }
    if (!ok) atomicAdd(unconverged, 1);
    double S = 0.0;
    for (int m = 0; m < k; ++m) S += exp(-beta * (dd[m] - dmin));
    for (int m = 0; m < k; ++m) cond[(size_t)i * k + m] = exp(-beta * (dd[m] - dmin)) / S;
}

// ---- symmetrisation
// extra[j] = number of rows i that list j while j does not list i; slot[e] = where i sits in j's list
// (-1 if it does not), kept for sym_fill (k <= 1280 fits 16 bits).  Sixteen lanes look one edge up: they
// read 64 contiguous bytes of row j at a time, so a row costs its three or four cache lines once.
__global__ __launch_bounds__(256) void sym_count(const int32_t *__restrict__ idx, int n, int k, int *__restrict__ extra,
                                                 int16_t *__restrict__ slot)
{
    const size_t e = global_index() >> 4;
    const int sub = (int)(threadIdx.x & 15u), grp = (int)((threadIdx.x & 63u) >> 4);
    const bool live = e < (size_t)n * k;
    const size_t ee = live ? e : 0;
    const int i = (int)(ee / k), j = idx[ee];
    const int32_t *r = idx + (size_t)j * k;
    int found = -1;
    for (int a0 = 0; a0 < k; a0 += 16) {
        const int a = a0 + sub;
        const bool hit = a < k && r[a] == i;
        const unsigned m = (unsigned)(__ballot(hit) >> (16 * grp)) & 0xFFFFu;
        if (m != 0u && found < 0) found = a0 + __builtin_ctz(m);
        if (__all(found >= 0)) break;
    }
    if (live && sub == 0) {
        slot[e] = (int16_t)found;
        if (found < 0) atomicAdd(&extra[j], 1);
    }
}

// row_ptr[i] = sum_{r<i} (k + extra[r]); single block, n up to 2^30
__global__ __launch_bounds__(1024) void sym_scan(const int *__restrict__ extra, int n, int k, int32_t *__restrict__ row_ptr,
                                                 int *__restrict__ cursor)
{
    __shared__ long long ws[16];
    const int per = (n + 1023) / 1024;
    const int s = threadIdx.x * per, e = min(n, s + per);
    long long a = 0;
    for (int i = s; i < e; ++i) a += k + extra[i];
    long long inc = a;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        long long t = __shfl_up(inc, o, WAVE);
        if (lane_id() >= o) inc += t;
    }
    if (lane_id() == WAVE - 1) ws[threadIdx.x >> 6] = inc;
    __syncthreads();
    long long base = 0;
    for (int q = 0; q < (int)(threadIdx.x >> 6); ++q) base += ws[q];
    long long pre = base + inc - a;
    for (int i = s; i < e; ++i) {
        row_ptr[i] = (int32_t)pre;
        cursor[i] = (int)pre + k;     // extras are appended after the row's own k entries
        pre += k + extra[i];
    }
    if (threadIdx.x == 1023) row_ptr[n] = (int32_t)pre;
}

__global__ __launch_bounds__(256) void sym_fill(const int32_t *__restrict__ idx, const double *__restrict__ cond, int n,
                                                int k, const int32_t *__restrict__ row_ptr, int *__restrict__ cursor,
                                                const int16_t *__restrict__ slots, int32_t *__restrict__ col,
                                                float *__restrict__ val)
{
    const size_t e = global_index();
    if (e >= (size_t)n * k) return;
    const int i = (int)(e / k), a = (int)(e % k), j = idx[e];
    const double pji = cond[e];
    const int slot = slots[e];
    const double pij = slot >= 0 ? cond[(size_t)j * k + slot] : 0.0;
    const float v = (float)((pji + pij) / (2.0 * (double)n));
    col[row_ptr[i] + a] = j;
    val[row_ptr[i] + a] = v;
    if (slot < 0) {
        const int pos = atomicAdd(&cursor[j], 1);
        col[pos] = i;
        val[pos] = v;
    }
}

// Sort each row by column.  Rows up to SORT_CAP entries: bitonic sort in LDS; longer rows: rank
// sort through global scratch.
__global__ __launch_bounds__(256) void sym_sort_rows(const int32_t *__restrict__ row_ptr, int n, int32_t *__restrict__ col,
                                                     float *__restrict__ val, uint64_t *__restrict__ scratch)
{
    __shared__ uint64_t s[SORT_CAP];
    if (global_block() >= (size_t)n) return;
    const int row = (int)global_block();
    const int b = row_ptr[row], len = row_ptr[row + 1] - b;
    if (len <= 1) return;
    if (len <= SORT_CAP) {
        int size = 1;
        while (size < len) size <<= 1;
        for (int t = threadIdx.x; t < size; t += blockDim.x)
            s[t] = t < len ? (((uint64_t)(uint32_t)col[b + t] << 32) | __float_as_uint(val[b + t])) : ~0ull;
        __syncthreads();
        bitonic_sort(s, size);
        for (int t = threadIdx.x; t < len; t += blockDim.x) {
            col[b + t] = (int32_t)(s[t] >> 32);
            val[b + t] = __uint_as_float((uint32_t)s[t]);
        }
    } else {
        uint64_t *tmp = scratch + b;
        for (int t = threadIdx.x; t < len; t += blockDim.x)
            tmp[t] = ((uint64_t)(uint32_t)col[b + t] << 32) | __float_as_uint(val[b + t]);
        __syncthreads();
        for (int t = threadIdx.x; t < len; t += blockDim.x) {
            const uint64_t me = tmp[t];
            int r = 0;
            for (int q = 0; q < len; ++q) r += tmp[q] < me;
            col[b + r] = (int32_t)(me >> 32);
            val[b + r] = __uint_as_float((uint32_t)me);
        }
    }
}

__global__ void max_norm_k(const float *__restrict__ norms, int n, float *__restrict__ out)
{
    __shared__ float ws[16];
    float m = 0.f;
    for (int i = threadIdx.x; i < n; i += blockDim.x) m = fmaxf(m, norms[i]);
    m = wave_max(m);
    if (lane_id() == 0) ws[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int q = 1; q < (int)(blockDim.x >> 6); ++q) m = fmaxf(m, ws[q]);
        *out = m;
    }
}

__global__ void d2_to_float(const double *__restrict__ in, float *__restrict__ out, size_t m)
{
    size_t i = global_index();
    if (i < m) out[i] = (float)in[i];
}

// ---- Eq. (10)-(11) for long rows on the same tiles: helpers of ivf_search_tiles() below
// the probed lists of every row, rows in list order
__global__ void probe_gather(const int32_t *__restrict__ probe, const int *__restrict__ lorder, int n, int tau, int nlist,
                             int32_t *__restrict__ probe_l)
{
    const size_t e = global_index();
    if (e >= (size_t)n * tau) return;
    const size_t pos = e / tau;
    const int r = (int)(e % tau);
    const int row = min(max(lorder[pos], 0), n - 1);
    probe_l[e] = min(max(probe[(size_t)row * tau + r], 0), nlist - 1);
}

// queries q0 .. q0 + rows of the pass, grouped by the list they probe at rank r
__global__ void rank_hist(const int32_t *__restrict__ probe_l, int q0, int rows, int tau, int r, int *__restrict__ bcnt)
{
    const size_t i = global_index();
    if (i < (size_t)rows) atomicAdd(&bcnt[probe_l[((size_t)q0 + i) * tau + r]], 1);
}

__global__ void rank_scatter(const int32_t *__restrict__ probe_l, int q0, int rows, int tau, int r,
                             const int *__restrict__ pairptr, int *__restrict__ bcur, int *__restrict__ pairq)
{
    const size_t i = global_index();
    if (i >= (size_t)rows) return;
    const int L = probe_l[((size_t)q0 + i) * tau + r];
    pairq[pairptr[L] + atomicAdd(&bcur[L], 1)] = q0 + (int)i;     // any order inside a list
}

// tiles of list L in the launch that takes rows chunk * DBC .. of every list
__global__ void tile_count(const int *__restrict__ pairptr, const int *__restrict__ cellptr, int nlist, int chunk, int tq,
                           int *__restrict__ tcnt)
{
    const int L = blockIdx.x * blockDim.x + threadIdx.x;
    if (L >= nlist) return;
    const int nq = pairptr[L + 1] - pairptr[L];
    const int rs = min(cellptr[L] + chunk * DBC, cellptr[L + 1]), re = min(cellptr[L + 1], rs + DBC);
    tcnt[L] = ((nq + tq - 1) / tq) * ((re - rs + TN - 1) / TN);
}

// out[i] = in[0] + .. + in[i-1], i = 0 .. m (one workgroup; the sums stay below 2^31 as the callers size things)
__global__ __launch_bounds__(1024) void excl_scan_k(const int *__restrict__ in, int m, int *__restrict__ out)
{
    __shared__ int ws[16];
    const int per = (m + 1023) / 1024;
    const int b = min((int)threadIdx.x * per, m), e = min(b + per, m);
    int a = 0;
    for (int i = b; i < e; ++i) a += in[i];
    int inc = a;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        const int t = __shfl_up(inc, o, WAVE);
        if (lane_id() >= o) inc += t;
    }
    if (lane_id() == WAVE - 1) ws[threadIdx.x >> 6] = inc;
    __syncthreads();
    int base = 0;
    for (int q = 0; q < (int)(threadIdx.x >> 6); ++q) base += ws[q];
    int pre = base + inc - a;
    for (int i = b; i < e; ++i) { const int v = in[i]; out[i] = pre; pre += v; }
    if (threadIdx.x == 1023) out[m] = pre;
}

// the evenly spaced sample of m of n rows: floor(i n / m)
__global__ void sample_rows_k(int *__restrict__ rows, int n, int m)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < m) rows[i] = (int)(((long long)i * n) / m);
}

__global__ void fill_int_k(int *__restrict__ a, int v, int m)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < m) a[i] = v;
}

// Queries without a certificate: exact distances to every row of their tau lists.  One workgroup per failed
// query f (row rows[f] of the list order): key t of its `stride` slots is the ordered distance to the t-th row
// of its lists taken in probe order, ids[t] that row's number in X; counts[f] = how many there are.
__global__ __launch_bounds__(256) void ivf_exact_keys(const float *__restrict__ X, int n, int d, const int *__restrict__ rows,
                                                      const int32_t *__restrict__ probe_l, int tau,
                                                      const int *__restrict__ cellptr, const int *__restrict__ lorder,
                                                      size_t stride, uint64_t *__restrict__ okey, int *__restrict__ ids,
                                                      int *__restrict__ counts)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *xi = reinterpret_cast<float *>(smem);
    const int f = blockIdx.x;
    const int pos = min(max(rows[f], 0), n - 1);
    const float *x = X + (size_t)min(max(lorder[pos], 0), n - 1) * d;
    for (int t = threadIdx.x; t < d; t += blockDim.x) xi[t] = x[t];
    __syncthreads();
    const int w = threadIdx.x >> 6;
    size_t off = 0;
    for (int r = 0; r < tau; ++r) {
        const int L = probe_l[(size_t)pos * tau + r];
        const int rs = cellptr[L], m = cellptr[L + 1] - rs;
        for (int u = w; u < m; u += 4) {
            if (off + u >= stride) break;
            const int row = min(max(lorder[rs + u], 0), n - 1);
            const float *y = X + (size_t)row * d;
            double sum = 0.0;
            for (int t = lane_id(); t < d; t += WAVE) { const double df = (double)xi[t] - (double)y[t]; sum += df * df; }
            sum = wave_sum(sum);
            if (lane_id() == 0) {
                okey[(size_t)f * stride + off + u] = rs + u == pos ? ~0ull : orderable64(sum);
                ids[(size_t)f * stride + off + u] = row;
            }
        }
        off += (size_t)m;
    }
    if (threadIdx.x == 0) counts[f] = (int)(off < stride ? off : stride);
}


struct Layout {
    float *norms, *norm_max, *tau;
    int *cnt, *fail_count, *fail_rows, *extra, *cursor, *unconv;
    float *mu;               // column means (d rounded up to SLAB)
    double *mu_part;         // their partial sums, MEAN_CHUNKS x d
    uint64_t *cand, *sort_scratch;
    uint16_t *xs;            // the split copy of X
    uint16_t *xh, *xsf;      // long rows: the high parts alone; the split copy of the rows of the second sweep
    float *norms_f;          // their norms
    int *fail2_count, *fail2_rows;
    int *clist, *ccount;     // rows of the current query block that need compaction, and how many (two counters take turns)
    int32_t *knn_idx;
    double *knn_d2, *cond;
    int kp, cap;
};

int margin_kp(int n, int k)
{
    int kp = k + (k / 2 > 32 ? k / 2 : 32);
    if (kp > n - 1) kp = n - 1;
    return kp;
}

size_t carve(Layout *L, int n, int d, int k, char *base)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += up(bytes); return (void *)p; };
    const int kp = margin_kp(n, k);
    const int cap = kp + COMPACT_SLACK + COMPACT_EVERY * DBC;
    const size_t qb = (size_t)(n < QB ? n : QB);
    void *q;
    q = take(4 * (size_t)n); if (L) L->norms = (float *)q;
    q = take(4); if (L) L->norm_max = (float *)q;
    q = take(4 * qb); if (L) L->tau = (float *)q;
    q = take(4 * qb); if (L) L->cnt = (int *)q;
    q = take(4 * qb); if (L) L->clist = (int *)q;
    q = take(8); if (L) L->ccount = (int *)q;
    q = take(4); if (L) L->fail_count = (int *)q;
    q = take(4 * (size_t)n); if (L) L->fail_rows = (int *)q;
    q = take(4 * (size_t)n); if (L) L->extra = (int *)q;
    q = take(4 * (size_t)n); if (L) L->cursor = (int *)q;
    q = take(4); if (L) L->unconv = (int *)q;
    q = take(4 * (size_t)((d + SLAB - 1) / SLAB * SLAB)); if (L) L->mu = (float *)q;
    q = take(8 * (size_t)MEAN_CHUNKS * d); if (L) L->mu_part = (double *)q;
    q = take(8 * qb * cap); if (L) L->cand = (uint64_t *)q;
    q = take(8 * (size_t)2 * n * k); if (L) L->sort_scratch = (uint64_t *)q;
    q = take(4 * (size_t)n * k); if (L) L->knn_idx = (int32_t *)q;
    q = take(8 * (size_t)n * k); if (L) L->knn_d2 = (double *)q;
    q = take(8 * (size_t)n * k); if (L) L->cond = (double *)q;
    q = take(4 * (size_t)n * ((d + SLAB - 1) / SLAB * SLAB)); if (L) L->xs = (uint16_t *)q;
    if (d >= HIGH_FIRST_MIN_D) {
        q = take(2 * (size_t)n * ((d + 2 * SLAB - 1) / (2 * SLAB) * (2 * SLAB))); if (L) L->xh = (uint16_t *)q;
        q = take(4 * qb * ((d + SLAB - 1) / SLAB * SLAB)); if (L) L->xsf = (uint16_t *)q;
        q = take(4 * qb); if (L) L->norms_f = (float *)q;
        q = take(4); if (L) L->fail2_count = (int *)q;
        q = take(4 * (size_t)n); if (L) L->fail2_rows = (int *)q;
    }
    if (L) { L->kp = kp; L->cap = cap; }
    return off;
}

int check_args(int32_t n, int32_t d, int32_t k)
{
    if (n < 2 || d < 1 || k < 1 || k >= n) return TSNE_EINVAL;
    if (k + (k / 2 > 32 ? k / 2 : 32) > MAX_KP || d > 4096) return TSNE_EINVAL;
    if ((int64_t)2 * n * k > 0x7FFFFFFFll) return TSNE_EINVAL;
    return TSNE_OK;
}

}  // namespace

#define HIPCHK(call)                                      \
    do {                                                  \
        hipError_t e_ = (call);                           \
        if (e_ != hipSuccess) {                           \
            fprintf(stderr, "tsne_build_P: %s failed: %s\n", #call, hipGetErrorString(e_)); \
            return TSNE_EHIP;                             \
        }                                                 \
    } while (0)

// ---- Eq. (10)-(11) with a flat second stage, rows longer than the double-precision kernels like
// The k nearest of the points in a query's tau probed lists, found the way tsne_build_P finds neighbours among all
// points: candidates from bf16 matrix-core tiles on the centred rows (here the tiles of (queries probing a list) x
// (rows of the list), queries grouped by list once per probe rank), exact distances in double for the k' best,
// a certificate per query, and an exact pass over its lists for a query without one.  The result is Eq. (11)'s by
// (distance in double, row number).  probe: n x tau list numbers (Eq. (10)), lorder: the rows in list order,
// cellptr: where each list starts in it; max_list and max_cand (longest list, most rows in one query's lists) from the caller.
namespace {
// (the k-th and the (k + 16)-th neighbour of a point are much farther apart than the error of a tile distance)
int search_kp(int n, int k) { return k + 16 < n - 1 ? k + 16 : n - 1; }

struct TileSearchLayout {
    float *norms, *norm_max, *tau, *mu;
    double *mu_part;
    int *cnt, *clist, *ccount, *fail_count, *fail_rows, *bcnt, *bcur, *pairptr, *tcnt, *tptr, *pairq, *fcnt;
    int32_t *probe_l;
    uint64_t *cand;
    uint16_t *xs;
    size_t cand_bytes;
};
constexpr int TS_ROWS = 1 << 17;     // queries per pass

size_t ts_carve(TileSearchLayout *L, int n, int d, int k, int nlist, int tau, char *base)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += up(bytes); return (void *)p; };
    const int kp = search_kp(n, k);
    const size_t cap = (size_t)kp + COMPACT_SLACK + COMPACT_EVERY * DBC;
    const size_t qb = (size_t)(n < TS_ROWS ? n : TS_ROWS);
    const size_t dp = ((size_t)d + SLAB - 1) / SLAB * SLAB;
    void *q;
    q = take(4 * (size_t)n); if (L) L->norms = (float *)q;
    q = take(4); if (L) L->norm_max = (float *)q;
    q = take(4 * qb); if (L) L->tau = (float *)q;
    q = take(4 * dp); if (L) L->mu = (float *)q;
    q = take(8 * (size_t)MEAN_CHUNKS * d); if (L) L->mu_part = (double *)q;
    q = take(4 * qb); if (L) L->cnt = (int *)q;
    q = take(4 * qb); if (L) L->clist = (int *)q;
    q = take(8); if (L) L->ccount = (int *)q;
    q = take(4); if (L) L->fail_count = (int *)q;
    q = take(4 * (size_t)n); if (L) L->fail_rows = (int *)q;
    q = take(4 * ((size_t)nlist + 1)); if (L) L->bcnt = (int *)q;
    q = take(4 * ((size_t)nlist + 1)); if (L) L->bcur = (int *)q;
    q = take(4 * ((size_t)nlist + 1)); if (L) L->pairptr = (int *)q;
    q = take(4 * ((size_t)nlist + 1)); if (L) L->tcnt = (int *)q;
    q = take(4 * ((size_t)nlist + 1)); if (L) L->tptr = (int *)q;
    q = take(4 * qb); if (L) L->pairq = (int *)q;
    q = take(4 * (size_t)(2 * k > 1 ? 2 * k : 1)); if (L) L->fcnt = (int *)q;
    q = take(4 * (size_t)n * tau); if (L) L->probe_l = (int32_t *)q;
    q = take(4 * (size_t)n * dp); if (L) L->xs = (uint16_t *)q;
    // candidate buffers; afterwards the keys and row numbers of the exact pass (12 bytes a slot, at least one query's n slots)
    size_t cb = 8 * qb * cap;
    if (cb < 12 * (size_t)n) cb = 12 * (size_t)n;
    q = take(cb); if (L) { L->cand = (uint64_t *)q; L->cand_bytes = cb; }
    return off;
}
}  // namespace

int ivf_search_tiles(const float *X, int n, int d, int k, int nlist, int tau, const int32_t *probe, const int *lorder,
                     const int *cellptr, int max_list, long long max_cand, int32_t *knn_idx, double *knn_d2, void *ws,
                     size_t ws_bytes, hipStream_t s)
{
    if (check_args(n, d, k) != TSNE_OK || nlist < 1 || tau < 1 || max_list < 1 || max_cand < 1) return TSNE_EINVAL;
    if (ws_bytes < ts_carve(nullptr, n, d, k, nlist, tau, nullptr)) return TSNE_ENOSPC;
    TileSearchLayout L;
    ts_carve(&L, n, d, k, nlist, tau, (char *)ws);
    const int kp = search_kp(n, k), cap = kp + COMPACT_SLACK + COMPACT_EVERY * DBC;
    const int dp = (d + SLAB - 1) / SLAB * SLAB;
    const int rows_per_chunk = (n + MEAN_CHUNKS - 1) / MEAN_CHUNKS, nchunks_mu = (n + rows_per_chunk - 1) / rows_per_chunk;
    hipLaunchKernelGGL(col_mean_part, dim3((d + 63) / 64, nchunks_mu), dim3(256), 0, s, X, n, d, rows_per_chunk, L.mu_part);
    hipLaunchKernelGGL(col_mean_final, dim3((dp + 255) / 256), dim3(256), 0, s, L.mu_part, nchunks_mu, n, d, dp, L.mu);
    hipLaunchKernelGGL(row_norms, wide_grid((size_t)n * WAVE), dim3(256), 0, s, X, L.mu, n, d, lorder, n, L.norms);
    hipLaunchKernelGGL(split_bf16, wide_grid((size_t)n * dp), dim3(256), 0, s, X, L.mu, n, d, dp, lorder, n, L.xs);
    hipLaunchKernelGGL(max_norm_k, dim3(1), dim3(1024), 0, s, L.norms, n, L.norm_max);
    hipLaunchKernelGGL(probe_gather, wide_grid((size_t)n * tau), dim3(256), 0, s, probe, lorder, n, tau, nlist, L.probe_l);
    HIPCHK(hipMemsetAsync(L.fail_count, 0, 4, s));
    float norm_max = 0.f;
    HIPCHK(hipMemcpyAsync(&norm_max, L.norm_max, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    const size_t rerank_smem = up((size_t)d * 4) + 8 * (size_t)MAX_KP;
    const int nchunks = (max_list + DBC - 1) / DBC;
    const unsigned lb = (unsigned)((nlist + 1 + 255) / 256);
    for (int q0 = 0; q0 < n; q0 += TS_ROWS) {
        const int rows = n - q0 < TS_ROWS ? n - q0 : TS_ROWS;
        hipLaunchKernelGGL(knn_reset, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, rows, L.ccount);
        // an upper bound of the tiles of one launch: sum over the lists of ceil(queries / 128) x (DBC / TN)
        const unsigned bound = (unsigned)(((size_t)rows / 128 + (size_t)nlist + 1) * (DBC / TN));
        for (int r = 0; r < tau; ++r) {
            hipLaunchKernelGGL(fill_int_k, dim3(lb), dim3(256), 0, s, L.bcnt, 0, nlist + 1);
            hipLaunchKernelGGL(fill_int_k, dim3(lb), dim3(256), 0, s, L.bcur, 0, nlist + 1);
            hipLaunchKernelGGL(rank_hist, wide_grid((size_t)rows), dim3(256), 0, s, L.probe_l, q0, rows, tau, r, L.bcnt);
            hipLaunchKernelGGL(excl_scan_k, dim3(1), dim3(1024), 0, s, L.bcnt, nlist, L.pairptr);
            hipLaunchKernelGGL(rank_scatter, wide_grid((size_t)rows), dim3(256), 0, s, L.probe_l, q0, rows, tau, r, L.pairptr,
                               L.bcur, L.pairq);
            for (int c = 0; c < nchunks; ++c) {
                hipLaunchKernelGGL(tile_count, dim3(lb), dim3(256), 0, s, L.pairptr, cellptr, nlist, c, 128, L.tcnt);
                hipLaunchKernelGGL(excl_scan_k, dim3(1), dim3(1024), 0, s, L.tcnt, nlist, L.tptr);
                hipLaunchKernelGGL((knn_tile_mfma<2, true, true>), dim3(bound), dim3(256), 0, s, (const uint4 *)L.xs, dp, q0,
                                   q0 + rows, 0, 0, L.norms, L.tau, L.cnt, L.cand, cap, L.ccount, (const uint4 *)L.xs, L.norms, 1,
                                   (const int *)nullptr, L.tptr, nlist, L.pairptr, L.pairq, cellptr, c);
                const int force = r == tau - 1 && c == nchunks - 1 ? 1 : 0;
                hipLaunchKernelGGL(knn_compact_list, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, cap, kp, rows, force,
                                   L.clist, L.ccount);
                const unsigned cg = (unsigned)(rows < 4096 ? rows : 4096);
                if (kp <= 320)
                    hipLaunchKernelGGL((knn_compact<512, 128>), dim3(cg), dim3(128), 0, s, L.tau, L.cnt, L.cand, cap, kp, rows, L.clist, L.ccount);
                else if (kp <= 832)
                    hipLaunchKernelGGL((knn_compact<1024, 128>), dim3(cg), dim3(128), 0, s, L.tau, L.cnt, L.cand, cap, kp, rows, L.clist, L.ccount);
                else
                    hipLaunchKernelGGL((knn_compact<4096, 256>), dim3(cg), dim3(256), 0, s, L.tau, L.cnt, L.cand, cap, kp, rows, L.clist, L.ccount);
            }
        }
        hipLaunchKernelGGL(knn_rerank, dim3(rows), dim3(256), rerank_smem, s, X, n, d, lorder, X, n, lorder, lorder, (const int *)nullptr, q0,
                           rows, k, kp, 0x7FFFFFFF, tile_error_coeff(d, true), 0.0, L.norms, norm_max, L.tau, L.cnt, L.cand, cap, knn_idx, knn_d2, L.fail_count,
                           L.fail_rows);
        HIPCHK(hipGetLastError());
    }
    int nfail = 0;
    HIPCHK(hipMemcpyAsync(&nfail, L.fail_count, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    if (nfail > 0) {
        const size_t stride = (size_t)max_cand;
        size_t nb_max = L.cand_bytes / (12 * stride);
        if (nb_max > (size_t)(2 * k)) nb_max = (size_t)(2 * k);
        if (nb_max < 1) return TSNE_ENOSPC;
        uint64_t *okey = L.cand;
        int *ids = reinterpret_cast<int *>(okey + nb_max * stride);
        for (int f0 = 0; f0 < nfail; f0 += (int)nb_max) {
            const int nb = nfail - f0 < (int)nb_max ? nfail - f0 : (int)nb_max;
            hipLaunchKernelGGL(ivf_exact_keys, dim3(nb), dim3(256), up((size_t)d * 4), s, X, n, d, L.fail_rows + f0, L.probe_l, tau,
                               cellptr, lorder, stride, okey, ids, L.fcnt);
            hipLaunchKernelGGL(knn_exact_select, dim3(nb), dim3(1024), 0, s, okey, stride, 0, L.fcnt, ids, k, L.fail_rows + f0,
                               lorder, n, knn_idx, knn_d2);
            HIPCHK(hipGetLastError());
        }
    }
    return TSNE_OK;
}

// ---- Eq. (10) for long rows: the tau nearest centroids of m rows of X (all rows, or the evenly spaced sample
// floor(i n / m) that k-means works on), by (distance in double, centroid number).  The same scheme once more:
// candidates from the tiles (queries against centroids, both centred on X's column means), the tau + 32 best
// re-ranked in double, a certificate, and all centroids in double for a query without one.
namespace {
struct TileProbeLayout {
    float *norms_q, *norms_c, *norm_max, *tau, *mu;
    double *mu_part;
    int *cnt, *clist, *ccount, *fail_count, *fail_rows, *qrows;
    uint64_t *cand;
    uint16_t *xs, *cs;
    size_t cand_bytes;
};

// (centroids are far apart against the error of a tile distance: eight spare candidates certify nearly every query)
int probe_kp(int nlist, int tau) { return tau + 8 < nlist ? tau + 8 : nlist; }

size_t tp_carve(TileProbeLayout *L, int n, int d, int nlist, int tau, char *base)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += up(bytes); return (void *)p; };
    const size_t cap = (size_t)probe_kp(nlist, tau) + COMPACT_SLACK + COMPACT_EVERY * DBC;
    const size_t qb = (size_t)(n < TS_ROWS ? n : TS_ROWS);
    const size_t dp = ((size_t)d + SLAB - 1) / SLAB * SLAB;
    void *q;
    q = take(4 * (size_t)n); if (L) L->norms_q = (float *)q;
    q = take(4 * (size_t)nlist); if (L) L->norms_c = (float *)q;
    q = take(4); if (L) L->norm_max = (float *)q;
    q = take(4 * qb); if (L) L->tau = (float *)q;
    q = take(4 * dp); if (L) L->mu = (float *)q;
    q = take(8 * (size_t)MEAN_CHUNKS * d); if (L) L->mu_part = (double *)q;
    q = take(4 * qb); if (L) L->cnt = (int *)q;
    q = take(4 * qb); if (L) L->clist = (int *)q;
    q = take(8); if (L) L->ccount = (int *)q;
    q = take(4); if (L) L->fail_count = (int *)q;
    q = take(4 * (size_t)n); if (L) L->fail_rows = (int *)q;
    q = take(4 * (size_t)n); if (L) L->qrows = (int *)q;
    q = take(4 * (size_t)n * dp); if (L) L->xs = (uint16_t *)q;
    q = take(4 * (size_t)nlist * dp); if (L) L->cs = (uint16_t *)q;
    size_t cb = 8 * qb * cap;
    if (cb < 8 * (size_t)nlist) cb = 8 * (size_t)nlist;      // the exact pass: at least one query's keys
    q = take(cb); if (L) { L->cand = (uint64_t *)q; L->cand_bytes = cb; }
    return off;
}
}  // namespace

// workspace of ivf_probe_tiles and, if k > 0, of ivf_search_tiles, which run one after the other (0: not for these sizes)
size_t ivf_tiles_workspace(int n, int d, int k, int nlist, int tau)
{
    if (n < 2 || d < 1 || d > 4096 || nlist < 1 || tau < 1 || tau > nlist) return 0;
    size_t a = tp_carve(nullptr, n, d, nlist, tau, nullptr), b = 0;
    if (k > 0) {
        if (check_args(n, d, k) != TSNE_OK) return 0;
        b = ts_carve(nullptr, n, d, k, nlist, tau, nullptr);
    }
    return a > b ? a : b;
}

// reuse_queries: the workspace still holds the query side (column means, sample rows, norms and split copy) of the
// previous call, which had the same X, n, d and m (the rounds of k-means: only the centroids change).
int ivf_probe_tiles(const float *X, int n, int d, const float *C, int nlist, int tau, int m, int32_t *probe, void *ws,
                    size_t ws_bytes, hipStream_t s, int reuse_queries)
{
    if (n < 2 || d < 1 || d > 4096 || nlist < 1 || tau < 1 || tau > nlist || m < 1 || m > n) return TSNE_EINVAL;
    if (ws_bytes < tp_carve(nullptr, n, d, nlist, tau, nullptr)) return TSNE_ENOSPC;
    TileProbeLayout L;
    tp_carve(&L, n, d, nlist, tau, (char *)ws);
    const int kp = probe_kp(nlist, tau), cap = kp + COMPACT_SLACK + COMPACT_EVERY * DBC;
    const int dp = (d + SLAB - 1) / SLAB * SLAB;
    const int rows_per_chunk = (n + MEAN_CHUNKS - 1) / MEAN_CHUNKS, nchunks_mu = (n + rows_per_chunk - 1) / rows_per_chunk;
    const int *rowmap = m < n ? L.qrows : nullptr;
    if (!reuse_queries) {
        hipLaunchKernelGGL(col_mean_part, dim3((d + 63) / 64, nchunks_mu), dim3(256), 0, s, X, n, d, rows_per_chunk, L.mu_part);
        hipLaunchKernelGGL(col_mean_final, dim3((dp + 255) / 256), dim3(256), 0, s, L.mu_part, nchunks_mu, n, d, dp, L.mu);
        if (m < n) hipLaunchKernelGGL(sample_rows_k, dim3((m + 255) / 256), dim3(256), 0, s, L.qrows, n, m);
        hipLaunchKernelGGL(row_norms, wide_grid((size_t)m * WAVE), dim3(256), 0, s, X, L.mu, m, d, rowmap, n, L.norms_q);
        hipLaunchKernelGGL(split_bf16, wide_grid((size_t)m * dp), dim3(256), 0, s, X, L.mu, m, d, dp, rowmap, n, L.xs);
    }
    hipLaunchKernelGGL(row_norms, wide_grid((size_t)nlist * WAVE), dim3(256), 0, s, C, L.mu, nlist, d, (const int *)nullptr, nlist,
                       L.norms_c);
    hipLaunchKernelGGL(split_bf16, wide_grid((size_t)nlist * dp), dim3(256), 0, s, C, L.mu, nlist, d, dp, (const int *)nullptr,
                       nlist, L.cs);
    hipLaunchKernelGGL(max_norm_k, dim3(1), dim3(1024), 0, s, L.norms_c, nlist, L.norm_max);
    HIPCHK(hipMemsetAsync(L.fail_count, 0, 4, s));
    float norm_max = 0.f;
    HIPCHK(hipMemcpyAsync(&norm_max, L.norm_max, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    const size_t rerank_smem = up((size_t)d * 4) + 8 * (size_t)MAX_KP;
    for (int q0 = 0; q0 < m; q0 += TS_ROWS) {
        const int rows = m - q0 < TS_ROWS ? m - q0 : TS_ROWS;
        hipLaunchKernelGGL(knn_reset, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, rows, L.ccount);
        // short first slabs bring the cut-offs down early (until a query has kp candidates it keeps every pair)
        int step = kp + 64 <= 256 ? 256 : DBC;
        for (int j0 = 0, jend; j0 < nlist; j0 = jend) {
            jend = j0 + step < nlist ? j0 + step : nlist;
            if (jend > step && step < DBC) step *= 2;
            const unsigned gy = (unsigned)((jend - j0 + TN - 1) / TN);
            const int force = jend >= nlist ? 1 : 0;
            if (d > KFLUSH)
                hipLaunchKernelGGL((knn_tile_mfma<2, true, false>), dim3((rows + 127) / 128, gy), dim3(256), 0, s,
                                   (const uint4 *)L.xs, dp, q0, q0 + rows, j0, jend, L.norms_q, L.tau, L.cnt, L.cand, cap, L.ccount,
                                   (const uint4 *)L.cs, L.norms_c, 0, (const int *)nullptr, (const int *)nullptr, 0,
                                   (const int *)nullptr, (const int *)nullptr, (const int *)nullptr, 0);
            else
                hipLaunchKernelGGL((knn_tile_mfma<KNN_MB, false, false>), dim3((rows + 64 * KNN_MB - 1) / (64 * KNN_MB), gy), dim3(256),
                                   0, s, (const uint4 *)L.xs, dp, q0, q0 + rows, j0, jend, L.norms_q, L.tau, L.cnt, L.cand, cap,
                                   L.ccount, (const uint4 *)L.cs, L.norms_c, 0, (const int *)nullptr, (const int *)nullptr, 0,
                                   (const int *)nullptr, (const int *)nullptr, (const int *)nullptr, 0);
            hipLaunchKernelGGL(knn_compact_list, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, cap, kp, rows, force,
                               L.clist, L.ccount);
            const unsigned cg = (unsigned)(rows < 4096 ? rows : 4096);
            hipLaunchKernelGGL((knn_compact<512, 128>), dim3(cg), dim3(128), 0, s, L.tau, L.cnt, L.cand, cap, kp, rows, L.clist,
                               L.ccount);
        }
        hipLaunchKernelGGL(knn_rerank, dim3(rows), dim3(256), rerank_smem, s, X, n, d, rowmap, C, nlist, (const int *)nullptr,
                           (const int *)nullptr, (const int *)nullptr, q0, rows, tau, kp, nlist, tile_error_coeff(d, d > KFLUSH), 0.0,
                           L.norms_q, norm_max, L.tau, L.cnt, L.cand, cap, probe,
                           (double *)nullptr, L.fail_count, L.fail_rows);
        HIPCHK(hipGetLastError());
    }
    int nfail = 0;
    HIPCHK(hipMemcpyAsync(&nfail, L.fail_count, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    if (nfail > 0) {
        size_t nb_max = L.cand_bytes / (8 * (size_t)nlist);
        if (nb_max > 4096) nb_max = 4096;
        if (nb_max < 1) return TSNE_ENOSPC;
        for (int f0 = 0; f0 < nfail; f0 += (int)nb_max) {
            const int nb = nfail - f0 < (int)nb_max ? nfail - f0 : (int)nb_max;
            hipLaunchKernelGGL(knn_exact_dists, wide_grid((size_t)nlist * WAVE), dim3(256), 0, s, X, n, rowmap, C, nlist, d,
                               L.fail_rows + f0, nb, 0, L.cand);
            hipLaunchKernelGGL(knn_exact_select, dim3(nb), dim3(1024), 0, s, L.cand, (size_t)nlist, nlist, (const int *)nullptr,
                               (const int *)nullptr, tau, L.fail_rows + f0, (const int *)nullptr, m, probe, (double *)nullptr);
            HIPCHK(hipGetLastError());
        }
    }
    return TSNE_OK;
}

extern "C" {

int tsne_build_P_workspace_bytes(int32_t n, int32_t d, int32_t k, size_t *bytes)
{
    if (!bytes || check_args(n, d, k) != TSNE_OK) return TSNE_EINVAL;
    *bytes = carve(nullptr, n, d, k, nullptr);
    return TSNE_OK;
}


// Alg. 1 line 2 from finished neighbour lists (L.knn_idx, L.knn_d2): Eq. (1) per row, then the symmetric CSR.
static int finish_P(const Layout &L, int32_t n, int32_t k, float perplexity, int32_t *d_row_ptr, int32_t *d_col,
                    float *d_val, int64_t cap_nnz, int64_t *nnz, int32_t *d_knn_idx, float *d_knn_d2,
                    int32_t *n_unconverged, hipStream_t s)
{
    const size_t nk = (size_t)n * k;
    const size_t ps_bytes = 64 * (size_t)(k | 1) * 8;
    const int ps_staged = ps_bytes <= 60 * 1024 ? 1 : 0;
    hipLaunchKernelGGL(perplexity_search, dim3((n + 63) / 64), dim3(64), ps_staged ? ps_bytes : 0, s, L.knn_d2, n, k,
                       log((double)perplexity), 1e-10, L.cond, L.unconv, ps_staged);
    // (the candidate buffers are free by now and hold 2 n k bytes with room to spare: 2 n k < 2^31 <= 8 * 65536 * 4160
    // for a full query block, and 2 k < 8 * 4160 for a short one)
    int16_t *slots = reinterpret_cast<int16_t *>(L.cand);
    hipLaunchKernelGGL(sym_count, wide_grid(nk * 16), dim3(256), 0, s, L.knn_idx, n, k, L.extra, slots);
    hipLaunchKernelGGL(sym_scan, dim3(1), dim3(1024), 0, s, L.extra, n, k, d_row_ptr, L.cursor);
    int32_t total = 0;
    HIPCHK(hipMemcpyAsync(&total, d_row_ptr + n, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    if ((int64_t)total > cap_nnz) return TSNE_ENOSPC;
    hipLaunchKernelGGL(sym_fill, wide_grid(nk), dim3(256), 0, s, L.knn_idx, L.cond, n, k, d_row_ptr,
                       L.cursor, slots, d_col, d_val);
    hipLaunchKernelGGL(sym_sort_rows, wide_grid((size_t)n * 256), dim3(256), 0, s, d_row_ptr, n, d_col, d_val, L.sort_scratch);
    if (d_knn_idx) HIPCHK(hipMemcpyAsync(d_knn_idx, L.knn_idx, 4 * nk, hipMemcpyDeviceToDevice, s));
    if (d_knn_d2)
        hipLaunchKernelGGL(d2_to_float, wide_grid(nk), dim3(256), 0, s, L.knn_d2, d_knn_d2, nk);
    int unconv = 0;
    HIPCHK(hipMemcpyAsync(&unconv, L.unconv, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    HIPCHK(hipGetLastError());
    *nnz = total;
    if (n_unconverged) *n_unconverged = unconv;
    return TSNE_OK;
}

int tsne_build_P(const float *d_X, int32_t n, int32_t d, float perplexity, int32_t k, int32_t *d_row_ptr,
                 int32_t *d_col, float *d_val, int64_t cap_nnz, int64_t *nnz, int32_t *d_knn_idx, float *d_knn_d2,
                 int32_t *n_unconverged, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!d_X || !d_row_ptr || !d_col || !d_val || !nnz || !d_workspace) return TSNE_EINVAL;
    if (check_args(n, d, k) != TSNE_OK) return TSNE_EINVAL;
    if (!(perplexity > 0.0f) || !(perplexity <= (float)k)) return TSNE_EINVAL;
    if (((uintptr_t)d_workspace % ALIGN) != 0) return TSNE_EINVAL;
    if (workspace_bytes < carve(nullptr, n, d, k, nullptr)) return TSNE_ENOSPC;
    hipStream_t s = (hipStream_t)stream;
    Layout L;
    carve(&L, n, d, k, (char *)d_workspace);
    const int kp = L.kp, cap = L.cap;

    const int dp = (d + SLAB - 1) / SLAB * SLAB;
    const int rows_per_chunk = (n + MEAN_CHUNKS - 1) / MEAN_CHUNKS, nchunks = (n + rows_per_chunk - 1) / rows_per_chunk;
    hipLaunchKernelGGL(col_mean_part, dim3((d + 63) / 64, nchunks), dim3(256), 0, s, d_X, n, d, rows_per_chunk, L.mu_part);
    hipLaunchKernelGGL(col_mean_final, dim3((dp + 255) / 256), dim3(256), 0, s, L.mu_part, nchunks, n, d, dp, L.mu);
    hipLaunchKernelGGL(row_norms, wide_grid((size_t)n * WAVE), dim3(256), 0, s, d_X, L.mu, n, d, (const int *)nullptr, n, L.norms);
    hipLaunchKernelGGL(split_bf16, wide_grid((size_t)n * dp), dim3(256), 0, s, d_X, L.mu, n, d, dp, (const int *)nullptr, n, L.xs);
    hipLaunchKernelGGL(max_norm_k, dim3(1), dim3(1024), 0, s, L.norms, n, L.norm_max);
    HIPCHK(hipMemsetAsync(L.fail_count, 0, 4, s));
    HIPCHK(hipMemsetAsync(L.unconv, 0, 4, s));
    HIPCHK(hipMemsetAsync(L.extra, 0, 4 * (size_t)n, s));
    float norm_max = 0.f;
    HIPCHK(hipMemcpyAsync(&norm_max, L.norm_max, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));

    // more LDS than a kernel may use by default
    HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&knn_tile_resident<1>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)resident_lds_bytes(1)));
    HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&knn_tile_resident<2>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)resident_lds_bytes(2)));
    HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void *>(&knn_tile_half), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)HALF_TILE_LDS));
    const size_t rerank_smem = up((size_t)d * 4) + 8 * (size_t)MAX_KP;
    const unsigned cgmax = 4096;
    auto compact = [&](int rows, const int *cc) {
        const unsigned cg = (unsigned)rows < cgmax ? (unsigned)rows : cgmax;
        if (kp <= 320)
            hipLaunchKernelGGL((knn_compact<512, 128>), dim3(cg), dim3(128), 0, s, L.tau, L.cnt, L.cand, cap, kp, rows, L.clist, cc);
        else if (kp <= 832)
            hipLaunchKernelGGL((knn_compact<1024, 128>), dim3(cg), dim3(128), 0, s, L.tau, L.cnt, L.cand, cap, kp, rows, L.clist, cc);
        else
            hipLaunchKernelGGL((knn_compact<4096, 256>), dim3(cg), dim3(256), 0, s, L.tau, L.cnt, L.cand, cap, kp, rows, L.clist, cc);
    };
    // Long rows: a first sweep with the high parts alone (a third of the matrix work, half the bytes, a coarser
    // bound: 2^-8 of the norms instead of 2^-16); its certificate still holds wherever the k-th and the k'-th
    // neighbour are farther apart than that, and only the rows it fails go through the three-product tiles.
    bool high_first = d >= HIGH_FIRST_MIN_D;
    const int dph = (d + 2 * SLAB - 1) / (2 * SLAB) * (2 * SLAB);
    float dot_scale = 1.0f;
    double e_add = 0.0;
    if (high_first) {
        HIPCHK(hipMemsetAsync(L.fail2_count, 0, 4, s));            // (borrowed for the largest magnitude)
        hipLaunchKernelGGL(max_abs_centred, dim3(2048), dim3(256), 0, s, d_X, L.mu, (size_t)n * d, d,
                           reinterpret_cast<unsigned int *>(L.fail2_count));
        float xmax = 0.f;
        HIPCHK(hipMemcpyAsync(&xmax, L.fail2_count, 4, hipMemcpyDeviceToHost, s));
        HIPCHK(hipStreamSynchronize(s));
        if (!(xmax > 0.f) || !(xmax < 1e15f)) {
            high_first = false;                                     // all rows equal, or values half precision cannot scale
        } else {
            int e = 0;
            (void)frexpf(xmax, &e);                                 // xmax < 2^e
            const float scale = ldexpf(1.0f, 15 - e);               // |x| scale < 2^15
            dot_scale = ldexpf(1.0f, 2 * (e - 15));
            // a scaled value below 2^-14 may be rounded to a subnormal half or flushed to zero: off by at most
            // delta = 2^-14 / scale per value, the dot product by delta (sum |q_t| + sum |x_t|) + D delta^2, the
            // distance by twice that; sum |x_t| <= sqrt(D) |x|
            const double delta = ldexp(1.0, -14) / (double)scale;
            e_add = 2.0 * (delta * 2.0 * sqrt((double)d) * sqrt((double)norm_max) + (double)d * delta * delta);
            hipLaunchKernelGGL(split_high, wide_grid((size_t)n * dph), dim3(256), 0, s, d_X, L.mu, n, d, dph, scale, L.xh);
        }
    }
    for (int q0 = 0; q0 < n; q0 += QB) {
        const int qend = q0 + QB < n ? q0 + QB : n, rows = qend - q0;
        hipLaunchKernelGGL(knn_reset, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, rows, L.ccount);
        // Until a row has k' candidates its cut-off is +inf and every pair is kept, and the pairs kept
        // right after are still many (a fraction k' / j0 of them).  Short first slabs get the cut-offs
        // down early: 256, 256, 512, 1024 rows, then DBC at a time.
        int step = kp + 64 <= 256 ? 256 : DBC;
        int launch = 0;
        for (int j0 = 0, jend; j0 < n; j0 = jend, ++launch) {
            jend = j0 + step < n ? j0 + step : n;
            if (jend > step && step < DBC) step *= 2;
            const unsigned gy = (unsigned)((jend - j0 + TN - 1) / TN);
            const int force = jend >= n ? 1 : 0;
            int *cc = L.ccount + (launch & 1), *cc_next = L.ccount + ((launch + 1) & 1);   // two lists take turns
            const bool resident = dp <= 2 * SLAB && rows >= RESIDENT_MIN_ROWS;
            if (resident) {
                if (dp == SLAB)
                    hipLaunchKernelGGL(knn_tile_resident<1>, dim3((rows + RQ - 1) / RQ), dim3(512), resident_lds_bytes(1), s,
                                       (const uint4 *)L.xs, q0, qend, j0, jend, L.norms, L.tau, L.cnt, L.cand, cap, kp, force,
                                       L.clist, cc, cc_next);
                else
                    hipLaunchKernelGGL(knn_tile_resident<2>, dim3((rows + RQ - 1) / RQ), dim3(512), resident_lds_bytes(2), s,
                                       (const uint4 *)L.xs, q0, qend, j0, jend, L.norms, L.tau, L.cnt, L.cand, cap, kp, force,
                                       L.clist, cc, cc_next);
            } else {
                if (high_first)
                    hipLaunchKernelGGL(knn_tile_half, dim3((unsigned)(8 * (((rows + HT - 1) / HT + 7) / 8) * ((jend - j0 + HT - 1) / HT))), dim3(HALF_THREADS),
                                       HALF_TILE_LDS, s, (const uint4 *)L.xh, dph, q0, qend, j0, jend, L.norms, L.tau, L.cnt, L.cand,
                                       cap, cc, dot_scale);
                else if (d > KFLUSH)
                    hipLaunchKernelGGL((knn_tile_mfma<2, true, false>), dim3((rows + 127) / 128, gy), dim3(256), 0, s,
                                       (const uint4 *)L.xs, dp, q0, qend, j0, jend, L.norms, L.tau, L.cnt, L.cand, cap, cc,
                                       (const uint4 *)L.xs, L.norms, 1, (const int *)nullptr, (const int *)nullptr, 0,
                                       (const int *)nullptr, (const int *)nullptr, (const int *)nullptr, 0);
                else
                    hipLaunchKernelGGL((knn_tile_mfma<KNN_MB, false, false>), dim3((rows + 64 * KNN_MB - 1) / (64 * KNN_MB), gy), dim3(256),
                                       0, s, (const uint4 *)L.xs, dp, q0, qend, j0, jend, L.norms, L.tau, L.cnt, L.cand, cap, cc,
                                       (const uint4 *)L.xs, L.norms, 1, (const int *)nullptr, (const int *)nullptr, 0,
                                       (const int *)nullptr, (const int *)nullptr, (const int *)nullptr, 0);
                // (the half-precision sweep, too, compacts every second launch only: a row that is not listed has room
                // for what two launches can append, and between the sweeps' 503-us launches the two small kernels of a
                // pass are 8 % of the time)
                if (high_first && !force && step >= DBC && launch % COMPACT_EVERY != COMPACT_EVERY - 1) continue;
                hipLaunchKernelGGL(knn_compact_list, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, cap, kp, rows, force,
                                   L.clist, cc);
            }
            // (every second slab after the resident kernel, where accepted pairs are cheap; the rows stay listed)
            if (resident && !force && step >= DBC && launch % COMPACT_EVERY != COMPACT_EVERY - 1) continue;
            compact(rows, cc);
        }
        hipLaunchKernelGGL(knn_rerank, dim3(rows), dim3(256), rerank_smem, s, d_X, n, d, (const int *)nullptr, d_X, n,
                           (const int *)nullptr, (const int *)nullptr, (const int *)nullptr, q0, rows, k, kp, n - 1,
                           high_first ? tile_error_coeff(d, false, true) : tile_error_coeff(d, d > KFLUSH), e_add, L.norms, norm_max,
                           L.tau, L.cnt, L.cand, cap, L.knn_idx, L.knn_d2, L.fail_count, L.fail_rows);
        HIPCHK(hipGetLastError());
    }
    int nfail = 0;
    HIPCHK(hipMemcpyAsync(&nfail, L.fail_count, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    const int *exact_rows = L.fail_rows;
    if (high_first && nfail > 0) {
        // second sweep: the rows the first one could not certify, QB at a time, as queries of their own (a split
        // copy of just these rows) against all rows
        HIPCHK(hipMemsetAsync(L.fail2_count, 0, 4, s));
        for (int f0 = 0; f0 < nfail; f0 += QB) {
            const int rows = nfail - f0 < QB ? nfail - f0 : QB;
            const int *fr = L.fail_rows + f0;
            hipLaunchKernelGGL(row_norms, wide_grid((size_t)rows * WAVE), dim3(256), 0, s, d_X, L.mu, rows, d, fr, n, L.norms_f);
            hipLaunchKernelGGL(split_bf16, wide_grid((size_t)rows * dp), dim3(256), 0, s, d_X, L.mu, rows, d, dp, fr, n, L.xsf);
            hipLaunchKernelGGL(knn_reset, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, rows, L.ccount);
            int step = kp + 64 <= 256 ? 256 : DBC;
            for (int j0 = 0, jend; j0 < n; j0 = jend) {
                jend = j0 + step < n ? j0 + step : n;
                if (jend > step && step < DBC) step *= 2;
                const unsigned gy = (unsigned)((jend - j0 + TN - 1) / TN);
                const int force = jend >= n ? 1 : 0;
                hipLaunchKernelGGL((knn_tile_mfma<2, true, false>), dim3((rows + 127) / 128, gy), dim3(256), 0, s,
                                   (const uint4 *)L.xsf, dp, 0, rows, j0, jend, L.norms_f, L.tau, L.cnt, L.cand, cap, L.ccount,
                                   (const uint4 *)L.xs, L.norms, 1, fr, (const int *)nullptr, 0, (const int *)nullptr,
                                   (const int *)nullptr, (const int *)nullptr, 0);
                hipLaunchKernelGGL(knn_compact_list, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, cap, kp, rows, force,
                                   L.clist, L.ccount);
                compact(rows, L.ccount);
            }
            hipLaunchKernelGGL(knn_rerank, dim3(rows), dim3(256), rerank_smem, s, d_X, n, d, fr, d_X, n, (const int *)nullptr, fr, fr,
                               0, rows, k, kp, n - 1, tile_error_coeff(d, true), 0.0, L.norms_f, norm_max, L.tau, L.cnt, L.cand, cap,
                               L.knn_idx, L.knn_d2, L.fail2_count, L.fail2_rows);
            HIPCHK(hipGetLastError());
        }
        HIPCHK(hipMemcpyAsync(&nfail, L.fail2_count, 4, hipMemcpyDeviceToHost, s));
        HIPCHK(hipStreamSynchronize(s));
        exact_rows = L.fail2_rows;
    }
    // Rows without a certificate (ties at the k-th distance, duplicates): exact distances to every row, 2k failed
    // rows a launch (their n keys each fit the space the symmetrisation sorts in later, 2 n k words).
    for (int f0 = 0; f0 < nfail; f0 += 2 * k) {
        const int nb = nfail - f0 < 2 * k ? nfail - f0 : 2 * k;
        hipLaunchKernelGGL(knn_exact_dists, wide_grid((size_t)n * WAVE), dim3(256), 0, s, d_X, n, (const int *)nullptr, d_X, n, d,
                           exact_rows + f0, nb, 1, L.sort_scratch);
        hipLaunchKernelGGL(knn_exact_select, dim3(nb), dim3(1024), 0, s, L.sort_scratch, (size_t)n, n, (const int *)nullptr,
                           (const int *)nullptr, k, exact_rows + f0, (const int *)nullptr, n, L.knn_idx, L.knn_d2);
        HIPCHK(hipGetLastError());
    }
    return finish_P(L, n, k, perplexity, d_row_ptr, d_col, d_val, cap_nnz, nnz, d_knn_idx, d_knn_d2, n_unconverged, s);
}

static int approx_lists(int32_t n, int32_t nlist)
{
    if (nlist > 0) return nlist;
    int v = (int)llround(sqrt((double)n));     // Sec. III-B: |C| = sqrt(N)
    if (v < 1) v = 1;
    if (v > 65536) v = 65536;
    return v;
}

constexpr int PQ_KSUB = 256;     // centroids per sub-quantiser: one code byte per sub-vector

int tsne_build_P_approx_workspace_bytes(int32_t n, int32_t d, int32_t k, int32_t nlist, int32_t tau, int32_t pq_m,
                                        size_t *bytes)
{
    if (!bytes || check_args(n, d, k) != TSNE_OK || pq_m < 0) return TSNE_EINVAL;
    nlist = approx_lists(n, nlist);
    const int tau_max = nlist < 32 ? nlist : 32;
    size_t ivf = 0, ivf_max = 0;
    // (room for the search to be repeated with more lists, see tsne_build_P_approx)
    if (pq_m > 0) {
        const int ksub = n < PQ_KSUB ? n : PQ_KSUB;
        if (tsne_ivfpq_workspace_bytes(n, d, k, nlist, tau, pq_m, ksub, &ivf) != TSNE_OK) return TSNE_EINVAL;
        if (tsne_ivfpq_workspace_bytes(n, d, k, nlist, tau_max, pq_m, ksub, &ivf_max) != TSNE_OK) return TSNE_EINVAL;
        const size_t coarse = ivf_workspace(n, d, 0, nlist, 1);       // training the coarse centroids comes first
        if (coarse > ivf) ivf = coarse;
    } else {
        if (tsne_ivf_workspace_bytes(n, d, k, nlist, tau, &ivf) != TSNE_OK) return TSNE_EINVAL;
        if (tsne_ivf_workspace_bytes(n, d, k, nlist, tau_max, &ivf_max) != TSNE_OK) return TSNE_EINVAL;
    }
    *bytes = carve(nullptr, n, d, k, nullptr) + up(4 * (size_t)nlist * d) + up(4 * (size_t)PQ_KSUB * d) +
             (ivf_max > ivf ? ivf_max : ivf);
    return TSNE_OK;
}

int tsne_build_P_approx(const float *d_X, int32_t n, int32_t d, float perplexity, int32_t k, int32_t nlist, int32_t tau,
                        int32_t kmeans_iters, int32_t pq_m, int32_t *d_row_ptr, int32_t *d_col, float *d_val, int64_t cap_nnz,
                        int64_t *nnz, int32_t *d_knn_idx, float *d_knn_d2, int32_t *n_unconverged, int32_t *tau_used,
                        void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!d_X || !d_row_ptr || !d_col || !d_val || !nnz || !d_workspace || kmeans_iters < 0) return TSNE_EINVAL;
    if (check_args(n, d, k) != TSNE_OK) return TSNE_EINVAL;
    if (!(perplexity > 0.0f) || !(perplexity <= (float)k)) return TSNE_EINVAL;
    if (((uintptr_t)d_workspace % ALIGN) != 0) return TSNE_EINVAL;
    nlist = approx_lists(n, nlist);
    size_t need = 0;
    if (tsne_build_P_approx_workspace_bytes(n, d, k, nlist, tau, pq_m, &need) != TSNE_OK) return TSNE_EINVAL;
    if (workspace_bytes < need) return TSNE_ENOSPC;
    hipStream_t s = (hipStream_t)stream;
    Layout L;
    size_t off = carve(&L, n, d, k, (char *)d_workspace);
    float *centroids = (float *)((char *)d_workspace + off);
    off += up(4 * (size_t)nlist * d);
    float *codebooks = (float *)((char *)d_workspace + off);
    off += up(4 * (size_t)PQ_KSUB * d);
    const int ksub = n < PQ_KSUB ? n : PQ_KSUB;
    void *ivf_ws = (char *)d_workspace + off;
    const size_t ivf_bytes = workspace_bytes - off;
    HIPCHK(hipMemsetAsync(L.unconv, 0, 4, s));
    HIPCHK(hipMemsetAsync(L.extra, 0, 4 * (size_t)n, s));
    int rc = ivf_train_device(d_X, n, d, nlist, kmeans_iters, centroids, ivf_ws, ivf_bytes, s);
    if (rc != TSNE_OK) return rc;
    if (pq_m > 0) {     // Eq. (8): the second-stage codebooks, one code byte per sub-vector
        rc = tsne_ivfpq_train(d_X, n, d, centroids, nlist, pq_m, ksub, kmeans_iters, codebooks, ivf_ws, ivf_bytes, s);
        if (rc != TSNE_OK) return rc;
    }
    // a row that finds fewer than k other points in its tau lists: twice the lists for everybody, and again
    const int tau_max = nlist < 32 ? nlist : 32;
    for (;;) {
        rc = pq_m > 0 ? tsne_ivfpq_knn(d_X, n, d, centroids, nlist, codebooks, pq_m, ksub, tau, k, L.knn_idx, L.knn_d2, ivf_ws,
                                       ivf_bytes, s)
                      : ivf_knn_device(d_X, n, d, centroids, nlist, tau, k, L.knn_idx, L.knn_d2, ivf_ws, ivf_bytes, s);
        if (rc != TSNE_ENUM || tau >= tau_max) break;
        tau = 2 * tau < tau_max ? 2 * tau : tau_max;
    }
    if (rc != TSNE_OK) return rc;
    if (tau_used) *tau_used = tau;
    return finish_P(L, n, k, perplexity, d_row_ptr, d_col, d_val, cap_nnz, nnz, d_knn_idx, d_knn_d2, n_unconverged, s);
}

}  // extern "C"
