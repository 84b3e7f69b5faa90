// Approximate neighbour search of Sec. III-B: inverted file over a k-means coarse quantiser, with a
// flat second stage (Eq. 10-11 with q(y) = y) or the product-quantised one of Eq. (8): q(y) = q1(y) +
// q2(y - q1(y)), q2 = m sub-quantisers of ksub centroids over the sub-vectors of the residual.
//
//   ivf_probe        Eq. (10): for every point the tau nearest centroids (tau = 1: the quantiser q1)
//   kmeans_accum / kmeans_finish   Lloyd update: centroid = mean of its points
//   cell_hist / scan_counts / cell_scatter / gather_double   the inverted file: points grouped by list
//   pair_hist / scan_counts / pair_scatter   (query, probed list) pairs grouped by list
//   ivf_score        squared distances of a list's points to the queries that probe it, kept as float keys
//   ivf_select       Eq. (11): the k smallest of a query's candidates, ordered by (distance, index)
//   residual_sub / pack_codes / ivfpq_score   the product quantiser: residual sub-vectors (training and
//                    encoding reuse the k-means and nearest-centroid kernels), codes, distances to the codes
//
// Every decision (nearest centroid, probed lists, the k nearest of the candidates) is taken on
// squared distances summed in double precision from the float inputs, ties towards the lower
// index, so the result is the definition's and does not depend on how the work is tiled.
//
// Distances are not a matrix product here: the work is N * tau * (points per list) * d, a percent
// or two of the exact search's, and its cost is in moving and selecting the distances as much as
// in forming them.  A wave takes 64 queries, one per lane, their coordinates in registers, against
// the rows of one list, which are the same for every lane and come through scalar loads; each lane
// keeps eight running sums.
#include "tsne_internal.h"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace {

constexpr size_t IVF_ALIGN = 256;
inline size_t up256(size_t v) { return (v + IVF_ALIGN - 1) / IVF_ALIGN * IVF_ALIGN; }

constexpr int IVF_DC = 64;       // coordinates per staged chunk
// Rows longer than this are searched on the matrix-core tiles; shorter ones by the double-precision kernels here, which
// are the faster ones there (benchmark stand-in at 64 coordinates: 0.22 s against 0.51 s through the tiles; 5M x 50 with
// 16 lists probed: 3.1 s against 14.2 s).
constexpr int TILES_MIN_D = IVF_DC;
constexpr int IVF_CB = 8;        // list rows per register block
constexpr int IVF_SAMPLE = 2048;      // keys of a row sampled for the cut
constexpr int IVF_BUF_MIN = 1024, IVF_BUF_MAX = 4096;   // keys that may pass the cut (3 k within these bounds)
constexpr int IVF_CCH = 256;          // list rows per tile of the distance kernel
constexpr int IVF_QW = 4;             // query groups of 64 (waves) per tile: they read the same list rows at about the same time
constexpr size_t IVF_D_MAX = (size_t)8 << 30;   // bytes of key scratch used at most

// ------------------------------------------------------------------ small helpers
// rows of d floats -> rows of dp doubles (dp = d rounded up to a multiple of four, the rest zero)
__global__ void to_double_k(const float *__restrict__ in, size_t rows, int d, int dp, double *__restrict__ out)
{
    size_t i = global_index();
    if (i >= rows * dp) return;
    const size_t r = i / dp;
    const int t = (int)(i % dp);
    out[i] = t < d ? (double)in[r * d + t] : 0.0;
}

__global__ void fill_i32_k(int *__restrict__ a, int v, size_t m)
{
    size_t i = global_index();
    if (i < m) a[i] = v;
}

__global__ void fill_u64_k(unsigned long long *__restrict__ a, size_t m)
{
    size_t i = global_index();
    if (i < m) a[i] = 0ull;
}

// ---- starting centroids, spread out: from the sample of m rows floor(j n / m) the first, then again and
// again the one farthest from those taken so far (squared distance in double, lowest j among equals)
__device__ __forceinline__ long long sample_row(int j, int n, int m) { return ((long long)j * n) / m; }

// mind[j] = min(mind[j], |sample j - sample sel[c]|^2); one wave per sample row
__global__ __launch_bounds__(256) void fps_update(const float *__restrict__ X, int n, int d, int m,
                                                  const int *__restrict__ sel, int c, double *__restrict__ mind, int first)
{
    const int j = blockIdx.x * 4 + (int)(threadIdx.x >> 6);
    if (j >= m) return;
    const float *x = X + (size_t)sample_row(j, n, m) * d;
    const float *y = X + (size_t)sample_row(sel[c], n, m) * d;
    double acc = 0.0;
    for (int t = lane_id(); t < d; t += WAVE) {
        const double df = (double)x[t] - (double)y[t];
        acc = fma(df, df, acc);
    }
    acc = wave_sum(acc);
    if (lane_id() == 0) mind[j] = first ? acc : fmin(mind[j], acc);
}

// sel[c] = argmax_j mind[j], lowest j among equals; one workgroup
__global__ __launch_bounds__(1024) void fps_argmax(const double *__restrict__ mind, int m, int *__restrict__ sel, int c)
{
    __shared__ double bv[1024];
    __shared__ int bi[1024];
    double v = -1.0;
    int idx = 0x7FFFFFFF;
    for (int j = threadIdx.x; j < m; j += 1024) {
        const double w = mind[j];
        if (w > v) { v = w; idx = j; }         // ascending j: a later equal value does not replace
    }
    bv[threadIdx.x] = v;
    bi[threadIdx.x] = idx;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            const double w = bv[threadIdx.x + o];
            const int wi = bi[threadIdx.x + o];
            if (w > bv[threadIdx.x] || (w == bv[threadIdx.x] && wi < bi[threadIdx.x])) { bv[threadIdx.x] = w; bi[threadIdx.x] = wi; }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) sel[c] = bi[0];
}

__global__ void fps_gather(const float *__restrict__ X, int n, int d, int m, int nlist, const int *__restrict__ sel,
                           float *__restrict__ C)
{
    size_t i = global_index();
    if (i >= (size_t)nlist * d) return;
    const int c = (int)(i / d), t = (int)(i % d);
    C[i] = X[(size_t)sample_row(sel[c], n, m) * d + t];
}

__global__ void max_abs_k(const float *__restrict__ X, size_t m, unsigned int *__restrict__ out)
{
    float v = 0.f;
    for (size_t i = global_index(); i < m; i += (size_t)gridDim.x * blockDim.x)
        v = fmaxf(v, fabsf(X[i]));
    v = wave_max(v);
    if (lane_id() == 0) atomicMax(out, __float_as_uint(v));   // non-negative floats order like their bits
}

// ------------------------------------------------------------------ the distance tile
// A lane keeps a chunk of IVF_DC coordinates of its own row in registers (zero past the end of the row).
__device__ __forceinline__ void load_chunk(float (&xr)[IVF_DC], const float *__restrict__ X, int d, int row, int t0, int tl)
{
    const float *src = X + (size_t)row * d + t0;
#pragma unroll
    for (int t = 0; t < IVF_DC; ++t) xr[t] = t < tl ? src[t] : 0.0f;
}

// The same for rows longer than one chunk, where the chunk is fetched again for every block of list rows:
// lane t reads coordinate t0 + t of each of the wave's 64 rows (contiguous across the lanes), the values go
// through this wave's 64 x 64 floats of LDS (slot of row r in line t: r ^ t) and come back one row per lane.
__device__ __forceinline__ void load_chunk_lds(float (&xr)[IVF_DC], float *xs, const float *__restrict__ X, int d,
                                               int myrow, int t0, int tl)
{
    const int lane = lane_id();
    __builtin_amdgcn_wave_barrier();      // (the reads of the previous chunk come first)
    for (int r0 = 0; r0 < WAVE; r0 += 16) {       // sixteen row loads in flight
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int row = __shfl(myrow, r0 + u);
            v[u] = lane < tl ? X[(size_t)row * d + t0 + lane] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) xs[lane * IVF_DC + ((r0 + u) ^ lane)] = v[u];
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int t = 0; t < IVF_DC; ++t) xr[t] = xs[t * IVF_DC + (lane ^ t)];
}

// acc[j] += sum over the chunk of (x_lane[t] - Y[row0 + j][t0 + t])^2; rows past row_last read row_last.
// Y has rows of dp doubles, dp a multiple of four with zeros past d, so whole groups of four can be taken;
// the rows are the same for every lane and arrive through scalar loads.
__device__ __forceinline__ void accumulate(double (&acc)[IVF_CB], float (&xr)[IVF_DC], const double *__restrict__ Y,
                                           int dp, int row0, int row_last, int t0, int tl)
{
    const double *y[IVF_CB];
#pragma unroll
    for (int j = 0; j < IVF_CB; ++j) {
        const int r = __builtin_amdgcn_readfirstlane(row0 + j < row_last ? row0 + j : row_last);
        y[j] = Y + (size_t)r * dp + t0;
    }
    // (The coordinates stay floats between the calls: widened once outside the caller's loop they would
    // take twice the registers and a wave slot per SIMD with them.)
#pragma unroll
    for (int t = 0; t < IVF_DC; ++t) asm volatile("" : "+v"(xr[t]));
#pragma unroll
    for (int t4 = 0; t4 < IVF_DC; t4 += 4) {
        if (t4 < tl) {
#pragma unroll
            for (int j = 0; j < IVF_CB; ++j) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const double df = (double)xr[t4 + u] - y[j][t4 + u];
                    acc[j] = fma(df, df, acc[j]);
                }
            }
        }
    }
}

// ------------------------------------------------------------------ Eq. (10)
// One wave per 64 consecutive points, one point per lane; the lane's tau best (distance, centroid)
// so far sit in LDS, ordered; centroids come in ascending index, so "strictly smaller" keeps the
// lower index among equals.
// LONG: rows longer than one chunk (the chunk buffer in LDS is there)
template <bool LONG>
__global__ __launch_bounds__(64) void ivf_probe(const float *__restrict__ X, int n, int d, int dp,
                                                const double *__restrict__ Cd, int nlist, int tau,
                                                int32_t *__restrict__ probe, int m)
{
    extern __shared__ __align__(16) unsigned char probe_dyn[];
    double *pd = reinterpret_cast<double *>(probe_dyn);
    int *pi = reinterpret_cast<int *>(probe_dyn + 8 * (size_t)WAVE * tau);
    float *xs = reinterpret_cast<float *>(probe_dyn + 12 * (size_t)WAVE * tau);   // present when d > IVF_DC
    const int lane = lane_id();
    // entry i of the output belongs to row floor(i n / m) of X: the m evenly spaced rows k-means works on,
    // or every row (m = n)
    const int i0 = blockIdx.x * WAVE;
    const int slot = min(i0 + lane, m - 1);
    const int i = (int)(((long long)slot * n) / m);
    float xr[IVF_DC];
    if (!LONG) load_chunk(xr, X, d, i, 0, d);
    int have = 0;
    double worst = INFINITY;
    // Long rows: a chunk of the coordinates serves four blocks of eight centroids before the next is fetched.
    constexpr int NSUB = LONG ? 4 : 1;
    for (int c0 = 0; c0 < nlist; c0 += NSUB * IVF_CB) {
        double acc[NSUB][IVF_CB];
#pragma unroll
        for (int u = 0; u < NSUB; ++u)
#pragma unroll
            for (int j = 0; j < IVF_CB; ++j) acc[u][j] = 0.0;
        for (int t0 = 0; t0 < d; t0 += IVF_DC) {
            const int tl = min(IVF_DC, d - t0);
            if (LONG) load_chunk_lds(xr, xs, X, d, i, t0, tl);
#pragma unroll
            for (int u = 0; u < NSUB; ++u)
                if (c0 + u * IVF_CB < nlist) accumulate(acc[u], xr, Cd, dp, c0 + u * IVF_CB, nlist - 1, t0, tl);
        }
#pragma unroll
        for (int u = 0; u < NSUB; ++u) {
#pragma unroll
            for (int j = 0; j < IVF_CB; ++j) {
                const int c = c0 + u * IVF_CB + j;
                const double v = acc[u][j];
                if (c < nlist && (have < tau || v < worst)) {
                    int s = have < tau ? have : tau - 1;
                    while (s > 0 && pd[(s - 1) * WAVE + lane] > v) {
                        pd[s * WAVE + lane] = pd[(s - 1) * WAVE + lane];
                        pi[s * WAVE + lane] = pi[(s - 1) * WAVE + lane];
                        --s;
                    }
                    pd[s * WAVE + lane] = v;
                    pi[s * WAVE + lane] = c;
                    if (have < tau) ++have;
                    if (have == tau) worst = pd[(tau - 1) * WAVE + lane];
                }
            }
        }
    }
    if (i0 + lane < m)
        for (int r = 0; r < tau; ++r) probe[(size_t)slot * tau + r] = pi[r * WAVE + lane];
}

// ------------------------------------------------------------------ Lloyd update
// Sums in fixed point (value * scale as a 64-bit integer): integer addition is associative, so the
// mean does not depend on the order in which the atomics land.
__global__ void kmeans_accum(const float *__restrict__ X, int n, int d, const int32_t *__restrict__ probe, int tau,
                             double scale, unsigned long long *__restrict__ sums, int *__restrict__ counts, int m)
{
    size_t idx = global_index();
    if (idx >= (size_t)m * d) return;
    const int i = (int)(idx / d), t = (int)(idx % d);
    const int c = probe[(size_t)i * tau];
    const size_t row = (size_t)(((long long)i * n) / m);       // the sample's i-th row
    atomicAdd(&sums[(size_t)c * d + t], (unsigned long long)llrint((double)X[row * d + t] * scale));
    if (t == 0) atomicAdd(&counts[c], 1);
}

__global__ void kmeans_finish(const unsigned long long *__restrict__ sums, const int *__restrict__ counts, int nlist,
                              int d, double inv_scale, float *__restrict__ C)
{
    size_t idx = global_index();
    if (idx >= (size_t)nlist * d) return;
    const int cnt = counts[idx / d];
    if (cnt > 0) C[idx] = (float)((double)(long long)sums[idx] * inv_scale / (double)cnt);   // an empty cell keeps its centroid
}

// ------------------------------------------------------------------ grouping by list
__global__ void cell_hist(const int32_t *__restrict__ probe, int n, int tau, int *__restrict__ cnt)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) atomicAdd(&cnt[probe[(size_t)i * tau]], 1);
}

// out[0] = 0, out[i + 1] = in[0] + .. + in[i]; with tiles != null also the same for the tiles of the distance
// kernel, ceil(in[i] / (64 IVF_QW)) * ceil(length of list i / IVF_CCH).  One workgroup.
__global__ __launch_bounds__(1024) void scan_counts(const int *__restrict__ in, int m, long long *__restrict__ out64,
                                                    int *__restrict__ out32, int *__restrict__ tiles,
                                                    const int *__restrict__ cellptr)
{
    __shared__ long long part[1024], tpart[1024];
    const int tid = threadIdx.x;
    const int chunk = (m + 1023) / 1024;
    const int b = min(tid * chunk, m), e = min(b + chunk, m);
    auto ntiles = [&](int i) -> long long {
        return (long long)((in[i] + IVF_QW * WAVE - 1) / (IVF_QW * WAVE)) * ((cellptr[i + 1] - cellptr[i] + IVF_CCH - 1) / IVF_CCH);
    };
    long long s = 0, ts = 0;
    for (int i = b; i < e; ++i) { s += in[i]; if (tiles) ts += ntiles(i); }
    part[tid] = s;
    tpart[tid] = ts;
    __syncthreads();
    if (tid == 0) {
        long long a = 0, ta = 0;
        for (int q = 0; q < 1024; ++q) {
            const long long v = part[q], tv = tpart[q];
            part[q] = a; tpart[q] = ta;
            a += v; ta += tv;
        }
        if (out64) out64[m] = a;
        if (out32) out32[m] = (int)a;
        if (tiles) tiles[m] = (int)(ta < 0x7FFFFFFFll ? ta : 0x7FFFFFFFll);
    }
    __syncthreads();
    s = part[tid];
    ts = tpart[tid];
    for (int i = b; i < e; ++i) {
        if (out64) out64[i] = s;
        if (out32) out32[i] = (int)s;
        if (tiles) { tiles[i] = (int)ts; ts += ntiles(i); }
        s += in[i];
    }
}

__global__ void cell_scatter(const int32_t *__restrict__ probe, int n, int tau, const int *__restrict__ cellptr,
                             int *__restrict__ cursor, int *__restrict__ lorder)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int c = probe[(size_t)i * tau];
    lorder[cellptr[c] + atomicAdd(&cursor[c], 1)] = i;   // the order inside a list does not matter to any result
}

__global__ void gather_double(const float *__restrict__ X, int n, int d, int dp, const int *__restrict__ lorder,
                              double *__restrict__ Xl)
{
    size_t idx = global_index();
    if (idx >= (size_t)n * dp) return;
    const size_t pos = idx / dp;
    const int t = (int)(idx % dp);
    Xl[idx] = t < d ? (double)X[(size_t)lorder[pos] * d + t] : 0.0;
}

// candidates a query sees: the sizes of its tau lists
__global__ void msize_k(const int32_t *__restrict__ probe, int n, int tau, const int *__restrict__ cellptr,
                        int *__restrict__ msize)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    int m = 0;
    for (int r = 0; r < tau; ++r) {
        const int c = probe[(size_t)i * tau + r];
        m += cellptr[c + 1] - cellptr[c];
    }
    msize[i] = m;
}

__global__ void pair_hist(const int32_t *__restrict__ probe, int qb, int rows, int tau, int *__restrict__ bcnt)
{
    size_t p = global_index();
    if (p < (size_t)rows * tau) atomicAdd(&bcnt[probe[(size_t)qb * tau + p]], 1);
}

__global__ void pair_scatter(const int32_t *__restrict__ probe, int qb, int rows, int tau,
                             const int *__restrict__ pairptr, int *__restrict__ bcur, int *__restrict__ pairq,
                             unsigned char *__restrict__ pairr)
{
    size_t p = global_index();
    if (p >= (size_t)rows * tau) return;
    const int B = probe[(size_t)qb * tau + p];
    const int pos = pairptr[B] + atomicAdd(&bcur[B], 1);
    pairq[pos] = qb + (int)(p / tau);
    pairr[pos] = (unsigned char)(p % tau);
}

// what is kept of a distance for the selection: the nearest float, finite (so that +inf can mark the query itself)
__device__ __forceinline__ float distance_key(double v) { return fminf((float)v, 3.4028234663852886e38f); }

// ------------------------------------------------------------------ distances of one list to the queries probing it
// A wave takes up to 64 (query, list) pairs of one list.  Lane's query q, the
// list its r-th: the distances go to the query's row of the scratch, after the sizes of its lists
// 0 .. r-1, in the list's order.  The query itself gets +inf.
template <bool LONG>
__global__ __launch_bounds__(IVF_QW * 64) void ivf_score(const float *__restrict__ X, int d, int dp, const double *__restrict__ Xl,
                                                const int *__restrict__ lorder, const int *__restrict__ cellptr,
                                                const int32_t *__restrict__ probe, int tau, int nlist,
                                                const int *__restrict__ pairptr, const int *__restrict__ tileptr,
                                                const int *__restrict__ pairq, const unsigned char *__restrict__ pairr,
                                                const long long *__restrict__ mprefix, long long base0,
                                                float *__restrict__ D)
{
    extern __shared__ __align__(16) float score_dyn[];     // a chunk buffer per wave, present when d > IVF_DC
    const int tile = blockIdx.x;
    if (tile >= tileptr[nlist]) return;
    int lo = 0, hi = nlist;            // last list whose first tile is <= tile and that has tiles
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tileptr[mid] <= tile) lo = mid; else hi = mid;
    }
    const int B = lo;
    const int lane = lane_id();
    // the list's tiles: IVF_QW query groups of 64, one per wave (fast index), times chunks of IVF_CCH of its rows
    const int qtiles = (pairptr[B + 1] - pairptr[B] + IVF_QW * WAVE - 1) / (IVF_QW * WAVE);
    const int within = tile - tileptr[B];
    const int chunk = within / qtiles;
    const int p0 = pairptr[B] + WAVE * (IVF_QW * (within - chunk * qtiles) + (int)(threadIdx.x >> 6));
    if (p0 >= pairptr[B + 1]) return;
    const int np = min(WAVE, pairptr[B + 1] - p0);
    const int p = p0 + min(lane, np - 1);
    const int q = pairq[p], r = pairr[p];
    long long off = mprefix[q] - base0;
    for (int rr = 0; rr < r; ++rr) {
        const int c = probe[(size_t)q * tau + rr];
        off += cellptr[c + 1] - cellptr[c];
    }
    float *dst = D + off;
    const int cb = cellptr[B], ce = min(cellptr[B + 1], cb + (chunk + 1) * IVF_CCH);
    float xr[IVF_DC];
    if (!LONG) load_chunk(xr, X, d, q, 0, d);
    constexpr int NSUB = LONG ? 4 : 1;     // blocks of eight list rows served by one fetch of a chunk
    for (int c0 = cb + chunk * IVF_CCH; c0 < ce; c0 += NSUB * IVF_CB) {
        double acc[NSUB][IVF_CB];
#pragma unroll
        for (int u = 0; u < NSUB; ++u)
#pragma unroll
            for (int j = 0; j < IVF_CB; ++j) acc[u][j] = 0.0;
        for (int t0 = 0; t0 < d; t0 += IVF_DC) {
            const int tl = min(IVF_DC, d - t0);
            if (LONG) load_chunk_lds(xr, score_dyn + (threadIdx.x >> 6) * (IVF_DC * WAVE), X, d, q, t0, tl);
#pragma unroll
            for (int u = 0; u < NSUB; ++u)
                if (c0 + u * IVF_CB < ce) accumulate(acc[u], xr, Xl, dp, c0 + u * IVF_CB, ce - 1, t0, tl);
        }
        if (lane < np) {
#pragma unroll
            for (int u = 0; u < NSUB; ++u)
#pragma unroll
                for (int j = 0; j < IVF_CB; ++j) {
                    const int c = c0 + u * IVF_CB + j;
                    if (c < ce) dst[c - cb] = lorder[c] == q ? INFINITY : distance_key(acc[u][j]);
                }
        }
    }
}

// ------------------------------------------------------------------ Eq. (11): the k smallest of a row
// What the distance kernel leaves per (query, candidate) is a float: the double sum rounded to nearest
// (monotone, so it orders like the sum, weakly) and kept finite, +inf standing for the query itself.
// The selection works on these keys and forms the sums again, with the same operations in the same
// order, for the few candidates whose exact value decides something.
__device__ __forceinline__ uint32_t key_bits(float f) { return __float_as_uint(f); }   // non-negative: ordered like the float
__device__ __forceinline__ bool pair_less(double da, int ia, double db, int ib) { return da < db || (da == db && ia < ib); }

// |x_q - x_j|^2 for rows q and j of X, summed like accumulate() does (which reads row j from the double
// copy: the same values, twice the bytes)
__device__ __forceinline__ double exact_d2(const float *__restrict__ X, int d, int q, int j)
{
    const float *x = X + (size_t)q * d;
    const float *y = X + (size_t)j * d;
    double acc = 0.0;
    for (int t = 0; t < d; ++t) {
        const double df = (double)x[t] - (double)y[t];
        acc = fma(df, df, acc);
    }
    return acc;
}

// The product-quantised second stage (Eq. 8): row id is stored as its list (q1) and m code bytes; codes == nullptr
// means the flat second stage.
struct PqView {
    const unsigned char *codes;   // n x m
    const float *cb;              // m x ksub x ds
    const float *C;               // the coarse centroids, nlist x d
    int m, ds, ksub;
};

// Eq. (11), |x_q - q(y)|^2 for y = row id stored in `list`: the query's residual to that list against the
// code's sub-vector centroids, every operation in double and none fused, each sub-vector's sum accumulated
// coordinate by coordinate and the m sums added in order.  The one function serves the distance kernel and
// the selection, so a candidate's value is the same bits wherever it is formed.
__device__ __forceinline__ double pq_d2(const float *__restrict__ X, int d, int q, int id, int list, const PqView &pq)
{
#pragma clang fp contract(off)
    const float *x = X + (size_t)q * d;
    const float *c = pq.C + (size_t)list * d;
    const unsigned char *code = pq.codes + (size_t)id * pq.m;
    double total = 0.0;
    for (int j = 0; j < pq.m; ++j) {
        const float *r = pq.cb + ((size_t)j * pq.ksub + min((int)code[j], pq.ksub - 1)) * pq.ds;
        double sub = 0.0;
        for (int t = 0; t < pq.ds; ++t) {
            const double rq = (double)x[j * pq.ds + t] - (double)c[j * pq.ds + t];
            const double df = rq - (double)r[t];
            const double sq = df * df;          // (a product and an addition: two roundings)
            sub = sub + sq;
        }
        total = total + sub;
    }
    return total;
}

// distance of candidate id to query q under the second stage in use (id's list is its nearest centroid,
// the first of its probes)
__device__ __forceinline__ double cand_d2(const float *__restrict__ X, int d, int q, int id,
                                          const int32_t *__restrict__ probe, int tau, const PqView &pq)
{
    return pq.codes ? pq_d2(X, d, q, id, probe[(size_t)id * tau], pq) : exact_d2(X, d, q, id);
}

// ------------------------------------------------------------------ product quantiser: residuals, codes, distances
// R[i][t] = x_i[j ds + t] - c[j ds + t], c the centroid of i's list: the j-th sub-vector of the residual (one
// float subtraction per coordinate), rows contiguous so that the k-means and nearest-centroid kernels take it as data
__global__ void residual_sub(const float *__restrict__ X, int n, int d, const float *__restrict__ C,
                             const int32_t *__restrict__ list, int j, int ds, float *__restrict__ R)
{
    const size_t e = global_index();
    if (e >= (size_t)n * ds) return;
    const size_t i = e / ds;
    const int t = (int)(e % ds);
    R[e] = X[i * d + (size_t)j * ds + t] - C[(size_t)list[i] * d + (size_t)j * ds + t];
}

__global__ void pack_codes(const int32_t *__restrict__ nearest, int n, int j, int m, unsigned char *__restrict__ codes)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) codes[(size_t)i * m + j] = (unsigned char)nearest[i];
}

// The distance kernel of the product-quantised second stage: same tiles and same places in the scratch as
// ivf_score; a lane's query against the codes of the list's rows, which are the same for every lane.
__global__ __launch_bounds__(IVF_QW * 64) void ivfpq_score(const float *__restrict__ X, int d, const int *__restrict__ lorder,
                                                  const int *__restrict__ cellptr, const int32_t *__restrict__ probe, int tau,
                                                  int nlist, const int *__restrict__ pairptr, const int *__restrict__ tileptr,
                                                  const int *__restrict__ pairq, const unsigned char *__restrict__ pairr,
                                                  const long long *__restrict__ mprefix, long long base0,
                                                  float *__restrict__ D, PqView pq)
{
    const int tile = blockIdx.x;
    if (tile >= tileptr[nlist]) return;
    int lo = 0, hi = nlist;            // last list whose first tile is <= tile and that has tiles
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tileptr[mid] <= tile) lo = mid; else hi = mid;
    }
    const int B = lo;
    const int lane = lane_id();
    const int qtiles = (pairptr[B + 1] - pairptr[B] + IVF_QW * WAVE - 1) / (IVF_QW * WAVE);
    const int within = tile - tileptr[B];
    const int chunk = within / qtiles;
    const int p0 = pairptr[B] + WAVE * (IVF_QW * (within - chunk * qtiles) + (int)(threadIdx.x >> 6));
    if (p0 >= pairptr[B + 1]) return;
    const int np = min(WAVE, pairptr[B + 1] - p0);
    const int p = p0 + min(lane, np - 1);
    const int q = pairq[p], r = pairr[p];
    long long off = mprefix[q] - base0;
    for (int rr = 0; rr < r; ++rr) {
        const int c = probe[(size_t)q * tau + rr];
        off += cellptr[c + 1] - cellptr[c];
    }
    float *dst = D + off;
    const int cb = cellptr[B], ce = min(cellptr[B + 1], cb + (chunk + 1) * IVF_CCH);
    for (int c = cb + chunk * IVF_CCH; c < ce; ++c) {
        const int id = lorder[c];
        const double v = pq_d2(X, d, q, id, B, pq);
        if (lane < np) dst[c - cb] = id == q ? INFINITY : distance_key(v);
    }
}

// The bucket of a 256-bin histogram that holds the need-th smallest element (1-based), how many of the
// elements wanted fall inside it, and its count.  All 256 threads call it after the histogram is complete.
__device__ __forceinline__ void find_bucket(const uint32_t *hist, int need, int *wtot, int *bucket, int *need_in,
                                            int *count)
{
    const int tid = threadIdx.x;
    const int h = (int)hist[tid];
    int tot;
    const int ex = wave_excl_scan(h, &tot);
    if (lane_id() == 0) wtot[tid >> 6] = tot;
    __syncthreads();
    int before = ex;
    for (int w = 0; w < (tid >> 6); ++w) before += wtot[w];
    if (before < need && need <= before + h) { *bucket = tid; *need_in = need - before; *count = h; }
    __syncthreads();
}

struct SelectShared {
    uint32_t hist[256];
    int wtot[4];
    int bucket, need, count;
};

// The rank-th smallest (1-based) of count 32-bit keys read through key(i); all 256 threads.  Returns the key;
// *need_in = how many of the rank smallest equal it, *equal = how many keys equal it.
template <typename KeyFn>
__device__ __forceinline__ uint32_t radix_kth(KeyFn key, int count, int rank, SelectShared &sh, int *need_in, int *equal)
{
    const int tid = threadIdx.x;
    uint32_t prefix = 0, mask = 0;
    int need = rank;
    for (int shift = 24; shift >= 0; shift -= 8) {
        sh.hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < count; i += 256) {
            const uint32_t kk = key(i);
            if ((kk & mask) == prefix) atomicAdd(&sh.hist[(kk >> shift) & 255u], 1u);
        }
        __syncthreads();
        find_bucket(sh.hist, need, sh.wtot, &sh.bucket, &sh.need, &sh.count);
        prefix |= (uint32_t)sh.bucket << shift;
        mask |= 255u << shift;
        need = sh.need;
        __syncthreads();
    }
    *need_in = need;
    *equal = sh.count;
    return prefix;
}

// One workgroup per query.  A strided sample of the row's keys gives a cut that, almost always, a few
// hundred keys pass, the k smallest among them: one sweep over the row collects those into LDS and the
// rest happens there.  If the cut fails (fewer than k keys, or more than the buffer holds) the k-th
// smallest key is found by sweeps over the whole row instead.  Keys below the k-th are in; the ones
// equal to it are ranked by (exact sum, index).
__global__ __launch_bounds__(256) void ivf_select(const float *__restrict__ F, const long long *__restrict__ mprefix,
                                                  long long base0, int qb, int tau, int k,
                                                  const int32_t *__restrict__ probe, const int *__restrict__ cellptr,
                                                  const int *__restrict__ lorder, const float *__restrict__ X, int d, int buf,
                                                  int32_t *__restrict__ knn_idx, double *__restrict__ knn_d2, PqView pq)
{
    extern __shared__ __align__(16) unsigned char sel_dyn[];
    double *wd = reinterpret_cast<double *>(sel_dyn);          // k winners, then up to buf equals
    int *wi = reinterpret_cast<int *>(wd + (k + buf));         // their indices; before that, their positions in the row
    uint32_t *bk = reinterpret_cast<uint32_t *>(wi + (k + buf));   // keys that passed the cut
    int *bp = reinterpret_cast<int *>(bk + buf);               // and their positions in the row
    uint32_t *sk = reinterpret_cast<uint32_t *>(wd + k);       // the sample (gone before the equals are written)
    __shared__ SelectShared sh;
    __shared__ int segoff[33], segbase[32];
    __shared__ int bcount, wcount, ecount;
    const int tid = threadIdx.x;
    const int q = qb + blockIdx.x;
    const float *src = F + (mprefix[q] - base0);
    const int M = (int)(mprefix[q + 1] - mprefix[q]);
    if (tid < tau) {
        const int c = probe[(size_t)q * tau + tid];
        segbase[tid] = cellptr[c];
        segoff[tid + 1] = cellptr[c + 1] - cellptr[c];
    }
    if (tid == 0) { segoff[0] = 0; bcount = 0; wcount = 0; ecount = 0; }
    __syncthreads();
    if (tid == 0)
        for (int r = 0; r < tau; ++r) segoff[r + 1] += segoff[r];
    __syncthreads();
    auto list_pos = [&](int pos) -> int {       // row position -> position in the list-ordered copy
        int r = 0;
        while (r + 1 < tau && pos >= segoff[r + 1]) ++r;
        return segbase[r] + pos - segoff[r];
    };
    int cnt = 0;
    bool direct;
    if (M <= buf) {
        for (int pos = tid; pos < M; pos += 256) { bk[pos] = key_bits(src[pos]); bp[pos] = pos; }
        cnt = M;
        direct = true;
        __syncthreads();
    } else {
        for (int j = tid; j < IVF_SAMPLE; j += 256) sk[j] = key_bits(src[(long long)j * M / IVF_SAMPLE]);
        __syncthreads();
        // about k S / M of the sample lie below the k-th key of the row; twice that and a dozen more is
        // more than three standard deviations above
        int r = 2 * (int)(((long long)k * IVF_SAMPLE + M - 1) / M) + 12;
        if (r > IVF_SAMPLE) r = IVF_SAMPLE;
        int dummy_need, dummy_equal;
        const uint32_t cut = radix_kth([&](int i) { return sk[i]; }, IVF_SAMPLE, r, sh, &dummy_need, &dummy_equal);
        for (int base = 0; base < M; base += 8 * 256) {     // eight loads in flight per thread
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int pos = base + u * 256 + tid;
                v[u] = pos < M ? src[pos] : INFINITY;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int pos = base + u * 256 + tid;
                const uint32_t kk = key_bits(v[u]);
                if (pos < M && kk <= cut) {
                    const int slot = atomicAdd(&bcount, 1);
                    if (slot < buf) { bk[slot] = kk; bp[slot] = pos; }
                }
            }
        }
        __syncthreads();
        cnt = bcount;
        direct = cnt >= k && cnt <= buf;
    }
    int need, equal;
    uint32_t Tf;
    if (direct) {
        Tf = radix_kth([&](int i) { return bk[i]; }, cnt, k, sh, &need, &equal);
    } else {
        Tf = radix_kth([&](int i) { return key_bits(src[i]); }, M, k, sh, &need, &equal);
        cnt = M;
    }
    const int less = k - need;                  // keys < Tf: all of them winners; keys == Tf: `equal` of them
    const bool small = equal <= buf;
    // positions of the winners (wi[0 .. less)) and of the equals (wi[k .. k + equal))
    for (int i = tid; i < cnt; i += 256) {
        const uint32_t kk = direct ? bk[i] : key_bits(src[i]);
        const int pos = direct ? bp[i] : i;
        if (kk < Tf) wi[atomicAdd(&wcount, 1)] = pos;
        else if (kk == Tf && small) wi[k + atomicAdd(&ecount, 1)] = pos;
    }
    __syncthreads();
    for (int a = tid; a < less + (small ? equal : 0); a += 256) {
        const int slot = a < less ? a : k + (a - less);
        const int id = lorder[list_pos(wi[slot])];
        wd[slot] = cand_d2(X, d, q, id, probe, tau, pq);
        wi[slot] = id;
    }
    __syncthreads();
    if (small) {
        // the `need` first of the equals by (sum, index)
        for (int a = tid; a < equal; a += 256) {
            const double da = wd[k + a];
            const int ia = wi[k + a];
            int rank = 0;
            for (int b = 0; b < equal; ++b) rank += pair_less(wd[k + b], wi[k + b], da, ia);
            if (rank < need) { wd[less + rank] = da; wi[less + rank] = ia; }
        }
    } else {
        // (More candidates at one float distance than the buffer holds: copies of one point.)  Among them
        // select on the bits of the exact sum, then on the index, a byte at a time, with sweeps over the row.
        unsigned long long p64 = 0, m64 = 0;
        int nd = need;
        for (int shift = 56; shift >= 0; shift -= 8) {
            sh.hist[tid] = 0;
            __syncthreads();
            for (int pos = tid; pos < M; pos += 256) {
                if (key_bits(src[pos]) != Tf) continue;
                const unsigned long long db =
                    (unsigned long long)__double_as_longlong(cand_d2(X, d, q, lorder[list_pos(pos)], probe, tau, pq));
                if ((db & m64) == p64) atomicAdd(&sh.hist[(unsigned)(db >> shift) & 255u], 1u);
            }
            __syncthreads();
            find_bucket(sh.hist, nd, sh.wtot, &sh.bucket, &sh.need, &sh.count);
            p64 |= (unsigned long long)sh.bucket << shift;
            m64 |= 255ull << shift;
            nd = sh.need;
            __syncthreads();
        }
        const int eq64 = sh.count;
        uint32_t pid = 0, mid = 0;
        uint32_t Tid = 0xFFFFFFFFu;
        if (nd < eq64) {
            int ni = nd;
            for (int shift = 24; shift >= 0; shift -= 8) {
                sh.hist[tid] = 0;
                __syncthreads();
                for (int pos = tid; pos < M; pos += 256) {
                    if (key_bits(src[pos]) != Tf) continue;
                    const uint32_t id = (uint32_t)lorder[list_pos(pos)];
                    if ((unsigned long long)__double_as_longlong(cand_d2(X, d, q, (int)id, probe, tau, pq)) != p64) continue;
                    if ((id & mid) == pid) atomicAdd(&sh.hist[(id >> shift) & 255u], 1u);
                }
                __syncthreads();
                find_bucket(sh.hist, ni, sh.wtot, &sh.bucket, &sh.need, &sh.count);
                pid |= (uint32_t)sh.bucket << shift;
                mid |= 255u << shift;
                ni = sh.need;
                __syncthreads();
            }
            Tid = pid;
        }
        for (int pos = tid; pos < M; pos += 256) {
            if (key_bits(src[pos]) != Tf) continue;
            const int id = lorder[list_pos(pos)];
            const double v = cand_d2(X, d, q, id, probe, tau, pq);
            const unsigned long long db = (unsigned long long)__double_as_longlong(v);
            if (db > p64) continue;
            if (db == p64 && (uint32_t)id > Tid) continue;
            const int slot = atomicAdd(&wcount, 1);
            wd[slot] = v;
            wi[slot] = id;
        }
    }
    __syncthreads();
    // final order by (distance, index)
    for (int a = tid; a < k; a += 256) {
        const double da = wd[a];
        const int ia = wi[a];
        int rank = 0;
        for (int b = 0; b < k; ++b) rank += pair_less(wd[b], wi[b], da, ia);
        knn_idx[(size_t)q * k + rank] = ia;
        knn_d2[(size_t)q * k + rank] = da;
    }
}

// LDS for the chunk buffers of the distance kernels: none while a row fits one chunk
size_t chunk_lds(int d, int waves) { return d > IVF_DC ? 4 * (size_t)IVF_DC * WAVE * waves : 0; }

// Eq. (10) for the rows floor(i n / m), i < m, of X.  Long rows go through the matrix-core tiles when the caller has
// their workspace (C: the centroids as floats); Cd: the centroids as doubles, rows padded to dp.
int launch_probe(const float *X, int n, int d, int dp, const double *Cd, int nlist, int tau, int32_t *probe, int m,
                 hipStream_t s, const float *C = nullptr, void *tiles_ws = nullptr, size_t tiles_bytes = 0,
                 int reuse_queries = 0)
{
    if (d > TILES_MIN_D && C && tiles_bytes > 0)
        return ivf_probe_tiles(X, n, d, C, nlist, tau, m, probe, tiles_ws, tiles_bytes, s, reuse_queries);
    const size_t lists = 12 * (size_t)WAVE * tau;
    if (d > IVF_DC)
        hipLaunchKernelGGL(ivf_probe<true>, dim3((m + WAVE - 1) / WAVE), dim3(WAVE), lists + chunk_lds(d, 1), s, X, n, d, dp, Cd,
                           nlist, tau, probe, m);
    else
        hipLaunchKernelGGL(ivf_probe<false>, dim3((m + WAVE - 1) / WAVE), dim3(WAVE), lists, s, X, n, d, dp, Cd, nlist, tau,
                           probe, m);
    return TSNE_OK;
}

int select_buf(int k)
{
    int b = 3 * k;
    if (b < IVF_BUF_MIN) b = IVF_BUF_MIN;
    if (b > IVF_BUF_MAX) b = IVF_BUF_MAX;
    return (b + 63) / 64 * 64;
}
size_t select_lds(int k, int buf) { return 12 * (size_t)(k + buf) + 8 * (size_t)buf; }

#define IVFCHK(call)                                      \
    do {                                                  \
        hipError_t e_ = (call);                           \
        if (e_ != hipSuccess) {                           \
            fprintf(stderr, "tsne ivf: %s failed: %s\n", #call, hipGetErrorString(e_)); \
            return TSNE_EHIP;                             \
        }                                                 \
    } while (0)

inline dim3 blocks(size_t m) { return wide_grid(m); }

struct IvfLayout {
    double *Cd, *Xl;
    float *D;
    int32_t *probe;
    int *cnt, *cellptr, *cursor, *lorder, *msize, *bcnt, *pairptr, *tileptr, *bcur, *pairq;
    unsigned char *pairr;
    long long *mprefix;
    unsigned long long *sums;
    unsigned int *maxabs;
    double *mind;
    int *sel;
    void *tiles_ws;          // workspace of the matrix-core search (long rows, flat second stage)
    size_t tiles_bytes;
    size_t d_bytes;
};

constexpr int IVF_BATCH_ROWS = 1 << 17;

// k_tiles: -1 none of the tile kernels is used with this workspace; 0 the probe only (k-means); > 0 the probe and a
// search for this k
size_t ivf_carve(IvfLayout *L, int n, int d, int nlist, int tau, char *base, size_t avail, int k_tiles = -1)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += up256(bytes); return (void *)p; };
    const size_t rows = (size_t)(n < IVF_BATCH_ROWS ? n : IVF_BATCH_ROWS);
    void *q;
    const size_t dp = ((size_t)d + 3) / 4 * 4;
    q = take(8 * (size_t)nlist * dp); if (L) L->Cd = (double *)q;
    q = take(8 * (size_t)n * dp); if (L) L->Xl = (double *)q;
    q = take(4 * (size_t)n * tau); if (L) L->probe = (int32_t *)q;
    q = take(4 * (size_t)(nlist + 1)); if (L) L->cnt = (int *)q;
    q = take(4 * (size_t)(nlist + 1)); if (L) L->cellptr = (int *)q;
    q = take(4 * (size_t)(nlist + 1)); if (L) L->cursor = (int *)q;
    q = take(4 * (size_t)n); if (L) L->lorder = (int *)q;
    q = take(4 * (size_t)n); if (L) L->msize = (int *)q;
    q = take(8 * (size_t)(n + 1)); if (L) L->mprefix = (long long *)q;
    q = take(4 * (size_t)(nlist + 1)); if (L) L->bcnt = (int *)q;
    q = take(4 * (size_t)(nlist + 1)); if (L) L->pairptr = (int *)q;
    q = take(4 * (size_t)(nlist + 1)); if (L) L->tileptr = (int *)q;
    q = take(4 * (size_t)(nlist + 1)); if (L) L->bcur = (int *)q;
    q = take(4 * rows * tau); if (L) L->pairq = (int *)q;
    q = take(rows * tau); if (L) L->pairr = (unsigned char *)q;
    q = take(8 * (size_t)nlist * d); if (L) L->sums = (unsigned long long *)q;
    q = take(4); if (L) L->maxabs = (unsigned int *)q;
    q = take(8 * 8 * (size_t)nlist); if (L) L->mind = (double *)q;
    q = take(4 * (size_t)nlist); if (L) L->sel = (int *)q;
    {
        const size_t tb = k_tiles >= 0 && d > TILES_MIN_D ? ivf_tiles_workspace(n, d, k_tiles, nlist, tau) : 0;
        q = take(tb); if (L) { L->tiles_ws = q; L->tiles_bytes = tb; }
    }
    // distance scratch: whatever is left, at least one row of n distances, at most IVF_D_MAX
    size_t want = 4 * (size_t)n * (size_t)(n < 4096 ? n : 4096);
    if (want > IVF_D_MAX) want = IVF_D_MAX;
    if (want < 4 * (size_t)n) want = 4 * (size_t)n;
    if (!base) return off + up256(want);
    size_t have = avail > off ? avail - off : 0;
    if (have > IVF_D_MAX) have = IVF_D_MAX;
    if (L) { L->D = (float *)(base + off); L->d_bytes = have / 8 * 8; }
    return off + up256(want);
}

int ivf_check(int n, int d, int k, int nlist, int tau)
{
    if (n < 2 || d < 1 || d > 4096 || k < 1 || k >= n || k > 1920) return TSNE_EINVAL;
    if (nlist < 1 || nlist > n || nlist > 65536 || tau < 1 || tau > 32 || tau > nlist) return TSNE_EINVAL;
    if ((int64_t)n * tau > 0x7FFFFFFFll) return TSNE_EINVAL;
    return TSNE_OK;
}

}  // namespace

size_t ivf_workspace(int n, int d, int k, int nlist, int tau)
{
    return ivf_carve(nullptr, n, d, nlist, tau, nullptr, 0, k);
}

// Lloyd's algorithm: `iters` rounds of (nearest centroid, mean of the members) from a spread-out start, on a sample
// of 256 rows per centroid.
int ivf_train_device(const float *X, int n, int d, int nlist, int iters, float *C, void *ws, size_t ws_bytes, hipStream_t s)
{
    IvfLayout L;
    if (ws_bytes < ivf_carve(nullptr, n, d, nlist, 1, nullptr, 0, 0)) return TSNE_ENOSPC;
    ivf_carve(&L, n, d, nlist, 1, (char *)ws, ws_bytes, 0);
    const size_t cd = (size_t)nlist * d, nd = (size_t)n * d;
    const int dp = (d + 3) / 4 * 4;
    {
        const int m = (long long)n < 8ll * nlist ? n : 8 * nlist;
        hipLaunchKernelGGL(fill_i32_k, dim3(1), dim3(256), 0, s, L.sel, 0, (size_t)1);       // the first sample row
        for (int c = 1; c < nlist; ++c) {
            hipLaunchKernelGGL(fps_update, dim3((m + 3) / 4), dim3(256), 0, s, X, n, d, m, L.sel, c - 1, L.mind, c == 1 ? 1 : 0);
            hipLaunchKernelGGL(fps_argmax, dim3(1), dim3(1024), 0, s, L.mind, m, L.sel, c);
        }
        hipLaunchKernelGGL(fps_gather, (blocks(cd)), dim3(256), 0, s, X, n, d, m, nlist, L.sel, C);
    }
    IVFCHK(hipMemsetAsync(L.maxabs, 0, 4, s));
    hipLaunchKernelGGL(max_abs_k, dim3(1024), dim3(256), 0, s, X, nd, L.maxabs);
    unsigned int bits = 0;
    IVFCHK(hipMemcpyAsync(&bits, L.maxabs, 4, hipMemcpyDeviceToHost, s));
    IVFCHK(hipStreamSynchronize(s));
    float xmax;
    memcpy(&xmax, &bits, 4);
    if (!(xmax < 1e38f)) return TSNE_EINVAL;
    // |sum| < n * xmax < 2^(ln + e): scale by 2^(62 - ln - e)
    int e = 0, ln = 0;
    if (xmax > 0.f) frexpf(xmax, &e);
    while ((1ll << ln) < (long long)n) ++ln;
    const double scale = ldexp(1.0, 62 - ln - e), inv_scale = ldexp(1.0, -(62 - ln - e));
    // the rounds work on min(n, 256 nlist) evenly spaced rows
    const int ms = (long long)n < 256ll * nlist ? n : 256 * nlist;
    for (int it = 0; it < iters; ++it) {
        hipLaunchKernelGGL(to_double_k, (blocks((size_t)nlist * dp)), dim3(256), 0, s, C, (size_t)nlist, d, dp, L.Cd);
        {
            const int rc = launch_probe(X, n, d, dp, L.Cd, nlist, 1, L.probe, ms, s, C, L.tiles_ws, L.tiles_bytes, it > 0);
            if (rc != TSNE_OK) return rc;
        }
        hipLaunchKernelGGL(fill_u64_k, (blocks(cd)), dim3(256), 0, s, L.sums, cd);
        hipLaunchKernelGGL(fill_i32_k, (blocks((size_t)nlist)), dim3(256), 0, s, L.cnt, 0, (size_t)nlist);
        hipLaunchKernelGGL(kmeans_accum, (blocks((size_t)ms * d)), dim3(256), 0, s, X, n, d, L.probe, 1, scale, L.sums, L.cnt,
                           ms);
        hipLaunchKernelGGL(kmeans_finish, (blocks(cd)), dim3(256), 0, s, L.sums, L.cnt, nlist, d, inv_scale, C);
    }
    IVFCHK(hipGetLastError());
    return TSNE_OK;
}

// Eq. (10)-(11): neighbour lists of every row of X from the inverted file over the centroids C.
static int ivf_knn_impl(const float *X, int n, int d, const float *C, int nlist, int tau, int k, int32_t *knn_idx,
                        double *knn_d2, void *ws, size_t ws_bytes, hipStream_t s, PqView pq)
{
    IvfLayout L;
    const int k_tiles = pq.codes ? -1 : k;
    if (ws_bytes < ivf_carve(nullptr, n, d, nlist, tau, nullptr, 0, k_tiles)) return TSNE_ENOSPC;
    ivf_carve(&L, n, d, nlist, tau, (char *)ws, ws_bytes, k_tiles);
    const int dp = (d + 3) / 4 * 4;
    hipLaunchKernelGGL(to_double_k, (blocks((size_t)nlist * dp)), dim3(256), 0, s, C, (size_t)nlist, d, dp, L.Cd);
    {
        const int rc = launch_probe(X, n, d, dp, L.Cd, nlist, tau, L.probe, n, s, C, L.tiles_ws, L.tiles_bytes);
        if (rc != TSNE_OK) return rc;
    }
    hipLaunchKernelGGL(fill_i32_k, (blocks((size_t)nlist + 1)), dim3(256), 0, s, L.cnt, 0, (size_t)nlist + 1);
    hipLaunchKernelGGL(fill_i32_k, (blocks((size_t)nlist + 1)), dim3(256), 0, s, L.cursor, 0, (size_t)nlist + 1);
    hipLaunchKernelGGL(cell_hist, (blocks((size_t)n)), dim3(256), 0, s, L.probe, n, tau, L.cnt);
    hipLaunchKernelGGL(scan_counts, dim3(1), dim3(1024), 0, s, L.cnt, nlist, (long long *)nullptr, L.cellptr, (int *)nullptr,
                       (const int *)nullptr);
    hipLaunchKernelGGL(cell_scatter, (blocks((size_t)n)), dim3(256), 0, s, L.probe, n, tau, L.cellptr, L.cursor, L.lorder);
    hipLaunchKernelGGL(gather_double, (blocks((size_t)n * dp)), dim3(256), 0, s, X, n, d, dp, L.lorder, L.Xl);
    hipLaunchKernelGGL(msize_k, (blocks((size_t)n)), dim3(256), 0, s, L.probe, n, tau, L.cellptr, L.msize);
    hipLaunchKernelGGL(scan_counts, dim3(1), dim3(1024), 0, s, L.msize, n, L.mprefix, (int *)nullptr, (int *)nullptr,
                       (const int *)nullptr);
    long long *mp = (long long *)malloc(8 * ((size_t)n + 1));
    if (!mp) return TSNE_ENOSPC;
    hipError_t e = hipMemcpyAsync(mp, L.mprefix, 8 * ((size_t)n + 1), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) { free(mp); return TSNE_EHIP; }
    long long mmax = 0;
    int rc = TSNE_OK;
    for (int i = 0; i < n; ++i) {
        const long long m = mp[i + 1] - mp[i];
        if (m - 1 < k) rc = TSNE_ENUM;            // fewer than k other points in the probed lists
        if (m > mmax) mmax = m;
    }
    if (rc == TSNE_OK && !pq.codes && d > TILES_MIN_D && L.tiles_bytes > 0) {
        // long rows, flat second stage: the distances of Eq. (11) on the matrix-core tiles of the exact search
        free(mp);
        int *cp = (int *)malloc(4 * ((size_t)nlist + 1));
        if (!cp) return TSNE_ENOSPC;
        e = hipMemcpyAsync(cp, L.cellptr, 4 * ((size_t)nlist + 1), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        int max_list = 1;
        for (int c = 0; c < nlist; ++c) if (cp[c + 1] - cp[c] > max_list) max_list = cp[c + 1] - cp[c];
        free(cp);
        if (e != hipSuccess) return TSNE_EHIP;
        return ivf_search_tiles(X, n, d, k, nlist, tau, L.probe, L.lorder, L.cellptr, max_list, mmax, knn_idx, knn_d2,
                                L.tiles_ws, L.tiles_bytes, s);
    }
    const long long d_cap = (long long)(L.d_bytes / 4);
    if (rc == TSNE_OK && mmax > d_cap) rc = TSNE_ENOSPC;
    if (rc != TSNE_OK) { free(mp); return rc; }
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ivf_score<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)chunk_lds(IVF_DC + 1, IVF_QW));
    if (e != hipSuccess) { free(mp); return TSNE_EHIP; }
    const int buf = select_buf(k);
    const size_t sel_bytes = select_lds(k, buf);
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ivf_select), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)select_lds(1920, IVF_BUF_MAX));
    if (e != hipSuccess) { free(mp); return TSNE_EHIP; }
    for (int qb = 0; qb < n;) {
        int qe = qb;
        while (qe < n && qe - qb < IVF_BATCH_ROWS && mp[qe + 1] - mp[qb] <= d_cap) ++qe;
        const int rows = qe - qb;
        const size_t pairs = (size_t)rows * tau;
        hipLaunchKernelGGL(fill_i32_k, (blocks((size_t)nlist + 1)), dim3(256), 0, s, L.bcnt, 0, (size_t)nlist + 1);
        hipLaunchKernelGGL(fill_i32_k, (blocks((size_t)nlist + 1)), dim3(256), 0, s, L.bcur, 0, (size_t)nlist + 1);
        hipLaunchKernelGGL(pair_hist, (blocks(pairs)), dim3(256), 0, s, L.probe, qb, rows, tau, L.bcnt);
        hipLaunchKernelGGL(scan_counts, dim3(1), dim3(1024), 0, s, L.bcnt, nlist, (long long *)nullptr, L.pairptr, L.tileptr,
                           L.cellptr);
        hipLaunchKernelGGL(pair_scatter, (blocks(pairs)), dim3(256), 0, s, L.probe, qb, rows, tau, L.pairptr, L.bcur,
                           L.pairq, L.pairr);
        int tiles = 0;
        e = hipMemcpyAsync(&tiles, L.tileptr + nlist, 4, hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess || tiles <= 0 || tiles == 0x7FFFFFFF) { free(mp); return e != hipSuccess ? TSNE_EHIP : TSNE_ENOSPC; }
        if (pq.codes)
            hipLaunchKernelGGL(ivfpq_score, dim3(tiles), dim3(IVF_QW * WAVE), 0, s, X, d, L.lorder, L.cellptr, L.probe, tau, nlist,
                               L.pairptr, L.tileptr, L.pairq, L.pairr, L.mprefix, mp[qb], L.D, pq);
        else if (d > IVF_DC)
            hipLaunchKernelGGL(ivf_score<true>, dim3(tiles), dim3(IVF_QW * WAVE), chunk_lds(d, IVF_QW), s, X, d, dp, L.Xl, L.lorder,
                               L.cellptr, L.probe, tau, nlist, L.pairptr, L.tileptr, L.pairq, L.pairr, L.mprefix, mp[qb], L.D);
        else
            hipLaunchKernelGGL(ivf_score<false>, dim3(tiles), dim3(IVF_QW * WAVE), 0, s, X, d, dp, L.Xl, L.lorder,
                               L.cellptr, L.probe, tau, nlist, L.pairptr, L.tileptr, L.pairq, L.pairr, L.mprefix, mp[qb], L.D);
        hipLaunchKernelGGL(ivf_select, dim3(rows), dim3(256), sel_bytes, s, L.D, L.mprefix, mp[qb], qb, tau, k, L.probe,
                           L.cellptr, L.lorder, X, d, buf, knn_idx, knn_d2, pq);
        qb = qe;
    }
    free(mp);
    IVFCHK(hipGetLastError());
    return TSNE_OK;
}

int ivf_knn_device(const float *X, int n, int d, const float *C, int nlist, int tau, int k, int32_t *knn_idx,
                   double *knn_d2, void *ws, size_t ws_bytes, hipStream_t s)
{
    PqView none;
    memset(&none, 0, sizeof(none));
    return ivf_knn_impl(X, n, d, C, nlist, tau, k, knn_idx, knn_d2, ws, ws_bytes, s, none);
}

// ---- product-quantised second stage
namespace {
struct PqLayout {
    int32_t *list, *nearest;      // q1 of every row; nearest sub-centroid of every row (one sub-quantiser at a time)
    float *R;                     // residual sub-vectors, n x ds
    double *cbd;                  // one sub-quantiser's centroids as doubles, ksub x (ds rounded up to 4)
    double *Cd;                   // the coarse centroids as doubles
    unsigned char *codes;         // n x m
    void *inner;                  // workspace of the calls made from here (k-means, the search)
    size_t inner_bytes;
};

int pq_check(int n, int d, int nlist, int m, int ksub)
{
    if (m < 1 || m > d || d % m != 0 || ksub < 1 || ksub > 256 || ksub > n) return TSNE_EINVAL;
    if (n < 1 || d < 1 || d > 4096 || nlist < 1 || nlist > n || nlist > 65536) return TSNE_EINVAL;
    return TSNE_OK;
}

size_t pq_carve(PqLayout *L, int n, int d, int k, int nlist, int tau, int m, int ksub, char *base, size_t avail)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += up256(bytes); return (void *)p; };
    const int ds = d / m, dsp = (ds + 3) / 4 * 4, dp = (d + 3) / 4 * 4;
    void *q;
    q = take(4 * (size_t)n); if (L) L->list = (int32_t *)q;
    q = take(4 * (size_t)n); if (L) L->nearest = (int32_t *)q;
    q = take(4 * (size_t)n * ds); if (L) L->R = (float *)q;
    q = take(8 * (size_t)ksub * dsp); if (L) L->cbd = (double *)q;
    q = take(8 * (size_t)nlist * dp); if (L) L->Cd = (double *)q;
    q = take((size_t)n * m); if (L) L->codes = (unsigned char *)q;
    size_t a = ivf_carve(nullptr, n, ds, ksub, 1, nullptr, 0, 0);         // training a sub-quantiser
    size_t b = tau > 0 ? ivf_carve(nullptr, n, d, nlist, tau, nullptr, 0) : 0;   // the search
    (void)k;
    if (L) { L->inner = base + off; L->inner_bytes = avail > off ? avail - off : 0; }
    return off + (a > b ? a : b);
}

// q1 of every row into L.list
void pq_lists(const float *X, int n, int d, const float *C, int nlist, PqLayout &L, hipStream_t s)
{
    const int dp = (d + 3) / 4 * 4;
    hipLaunchKernelGGL(to_double_k, (blocks((size_t)nlist * dp)), dim3(256), 0, s, C, (size_t)nlist, d, dp, L.Cd);
    launch_probe(X, n, d, dp, L.Cd, nlist, 1, L.list, n, s);
}
}  // namespace

extern "C" {

int tsne_ivfpq_workspace_bytes(int32_t n, int32_t d, int32_t k, int32_t nlist, int32_t tau, int32_t m, int32_t ksub,
                               size_t *bytes)
{
    if (!bytes || pq_check(n, d, nlist, m, ksub) != TSNE_OK || ivf_check(n, d, k, nlist, tau) != TSNE_OK) return TSNE_EINVAL;
    *bytes = pq_carve(nullptr, n, d, k, nlist, tau, m, ksub, nullptr, 0);
    return TSNE_OK;
}

int tsne_ivfpq_train(const float *d_X, int32_t n, int32_t d, const float *d_centroids, int32_t nlist, int32_t m,
                     int32_t ksub, int32_t iters, float *d_codebooks, void *d_workspace, size_t workspace_bytes,
                     void *stream)
{
    if (!d_X || !d_centroids || !d_codebooks || !d_workspace || iters < 0) return TSNE_EINVAL;
    if (pq_check(n, d, nlist, m, ksub) != TSNE_OK) return TSNE_EINVAL;
    if (((uintptr_t)d_workspace % IVF_ALIGN) != 0) return TSNE_EINVAL;
    if (workspace_bytes < pq_carve(nullptr, n, d, 1, nlist, 0, m, ksub, nullptr, 0)) return TSNE_ENOSPC;
    hipStream_t s = (hipStream_t)stream;
    PqLayout L;
    pq_carve(&L, n, d, 1, nlist, 0, m, ksub, (char *)d_workspace, workspace_bytes);
    const int ds = d / m;
    pq_lists(d_X, n, d, d_centroids, nlist, L, s);
    for (int j = 0; j < m; ++j) {
        hipLaunchKernelGGL(residual_sub, (blocks((size_t)n * ds)), dim3(256), 0, s, d_X, n, d, d_centroids, L.list, j, ds, L.R);
        const int rc = ivf_train_device(L.R, n, ds, ksub, iters, d_codebooks + (size_t)j * ksub * ds, L.inner, L.inner_bytes, s);
        if (rc != TSNE_OK) return rc;
    }
    IVFCHK(hipStreamSynchronize(s));
    IVFCHK(hipGetLastError());
    return TSNE_OK;
}

int tsne_ivfpq_knn(const float *d_X, int32_t n, int32_t d, const float *d_centroids, int32_t nlist,
                   const float *d_codebooks, int32_t m, int32_t ksub, int32_t tau, int32_t k, int32_t *d_knn_idx,
                   double *d_knn_d2, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!d_X || !d_centroids || !d_codebooks || !d_knn_idx || !d_knn_d2 || !d_workspace) return TSNE_EINVAL;
    if (pq_check(n, d, nlist, m, ksub) != TSNE_OK || ivf_check(n, d, k, nlist, tau) != TSNE_OK) return TSNE_EINVAL;
    if (((uintptr_t)d_workspace % IVF_ALIGN) != 0) return TSNE_EINVAL;
    if (workspace_bytes < pq_carve(nullptr, n, d, k, nlist, tau, m, ksub, nullptr, 0)) return TSNE_ENOSPC;
    hipStream_t s = (hipStream_t)stream;
    PqLayout L;
    pq_carve(&L, n, d, k, nlist, tau, m, ksub, (char *)d_workspace, workspace_bytes);
    const int ds = d / m, dsp = (ds + 3) / 4 * 4;
    // codes: for every sub-vector of the residual the nearest centroid of its sub-quantiser
    pq_lists(d_X, n, d, d_centroids, nlist, L, s);
    for (int j = 0; j < m; ++j) {
        hipLaunchKernelGGL(residual_sub, (blocks((size_t)n * ds)), dim3(256), 0, s, d_X, n, d, d_centroids, L.list, j, ds, L.R);
        hipLaunchKernelGGL(to_double_k, (blocks((size_t)ksub * dsp)), dim3(256), 0, s, d_codebooks + (size_t)j * ksub * ds,
                           (size_t)ksub, ds, dsp, L.cbd);
        launch_probe(L.R, n, ds, dsp, L.cbd, ksub, 1, L.nearest, n, s);
        hipLaunchKernelGGL(pack_codes, (blocks((size_t)n)), dim3(256), 0, s, L.nearest, n, j, m, L.codes);
    }
    PqView pq;
    pq.codes = L.codes; pq.cb = d_codebooks; pq.C = d_centroids; pq.m = m; pq.ds = ds; pq.ksub = ksub;
    const int rc = ivf_knn_impl(d_X, n, d, d_centroids, nlist, tau, k, d_knn_idx, d_knn_d2, L.inner, L.inner_bytes, s, pq);
    if (rc != TSNE_OK) return rc;
    IVFCHK(hipStreamSynchronize(s));
    return TSNE_OK;
}

int tsne_ivf_workspace_bytes(int32_t n, int32_t d, int32_t k, int32_t nlist, int32_t tau, size_t *bytes)
{
    if (!bytes || ivf_check(n, d, k, nlist, tau) != TSNE_OK) return TSNE_EINVAL;
    *bytes = ivf_workspace(n, d, k, nlist, tau);
    return TSNE_OK;
}

int tsne_ivf_train(const float *d_X, int32_t n, int32_t d, int32_t nlist, int32_t iters, float *d_centroids,
                   void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!d_X || !d_centroids || !d_workspace || iters < 0) return TSNE_EINVAL;
    if (n < 1 || d < 1 || d > 4096 || nlist < 1 || nlist > n || nlist > 65536) return TSNE_EINVAL;
    if (((uintptr_t)d_workspace % IVF_ALIGN) != 0) return TSNE_EINVAL;
    int rc = ivf_train_device(d_X, n, d, nlist, iters, d_centroids, d_workspace, workspace_bytes, (hipStream_t)stream);
    if (rc != TSNE_OK) return rc;
    IVFCHK(hipStreamSynchronize((hipStream_t)stream));
    return TSNE_OK;
}

int tsne_ivf_knn(const float *d_X, int32_t n, int32_t d, const float *d_centroids, int32_t nlist, int32_t tau, int32_t k,
                 int32_t *d_knn_idx, double *d_knn_d2, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!d_X || !d_centroids || !d_knn_idx || !d_knn_d2 || !d_workspace) return TSNE_EINVAL;
    if (ivf_check(n, d, k, nlist, tau) != TSNE_OK) return TSNE_EINVAL;
    if (((uintptr_t)d_workspace % IVF_ALIGN) != 0) return TSNE_EINVAL;
    int rc = ivf_knn_device(d_X, n, d, d_centroids, nlist, tau, k, d_knn_idx, d_knn_d2, d_workspace, workspace_bytes,
                            (hipStream_t)stream);
    if (rc != TSNE_OK) return rc;
    IVFCHK(hipStreamSynchronize((hipStream_t)stream));
    return TSNE_OK;
}

}  // extern "C"
