// Alg. 1 lines 1-2 of the paper on gfx950: the sparse affinity matrix P.
//
//   row_norms            |x_i|^2 in double, rounded to float
//   knn_tile_mfma        Sec. III-B, exact reading: all-pairs squared distances
//                        |q|^2 + |x|^2 - 2 q.x, the dot products on the matrix cores
//                        (v_mfma_f32_32x32x2_f32, 128x128 tiles through LDS).  The N x N matrix is
//                        never stored: the epilogue keeps a pair only if it beats the query row's
//                        current cut-off and appends it to that row's candidate buffer.
//   knn_compact          per query row, sorts the buffer, keeps the best k' = k + margin and lowers
//                        the cut-off to the k'-th distance
//   knn_rerank           recomputes the k' candidate distances as sum_t (x_it - x_jt)^2 in double,
//                        orders them by (distance, index), keeps k, and certifies the row: every
//                        discarded pair had a single-precision distance >= cut-off, so it cannot
//                        belong to the k nearest if cut-off - error bound > exact k-th distance
//   knn_exact_dists / knn_exact_select   rows that fail the certificate: all n distances in
//                        double, radix selection of the k-th smallest, ties by index
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
constexpr int MAX_KP = 1920;    // k' limit: k' + COMPACT_SLACK + DBC must fit the LDS sort
constexpr int SORT_CAP = 4096;  // candidate buffer entries per row = LDS sort size
constexpr int TM = 128, TN = 128, BK = 32, LDS_STRIDE = BK + 4;
constexpr int COMPACT_SLACK = 128; // new candidates per row that trigger a re-sort of its buffer
constexpr int KFLUSH = 64;      // columns summed on the matrix cores before a flush into the running sum

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

__global__ __launch_bounds__(256) void row_norms(const float *__restrict__ X, int n, int d, float *__restrict__ norms)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    const float *x = X + (size_t)row * d;
    double s = 0.0;
    for (int t = lane_id(); t < d; t += WAVE) { double v = (double)x[t]; s += v * v; }
    s = wave_sum(s);
    if (lane_id() == 0) norms[row] = (float)s;
}

__global__ void knn_reset(float *__restrict__ tau, int *__restrict__ cnt, int rows)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows) { tau[i] = INFINITY; cnt[i] = 0; }
}

// Loads a 128 x 32 slab of X (rows r0.., columns k0..) into registers as 4 float4 per thread;
// rows >= rend and columns >= d read as 0.
__device__ __forceinline__ void load_slab(const float *__restrict__ X, int d, int r0, int rend, int k0, bool vec,
                                          float4 v[4])
{
    const int kq = (threadIdx.x & 7) * 4;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int r = r0 + (threadIdx.x >> 3) + 32 * it;
        const int k = k0 + kq;
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < rend) {
            const float *p = X + (size_t)r * d + k;
            if (vec && k + 3 < d) a = *reinterpret_cast<const float4 *>(p);
            else {
                if (k < d) a.x = p[0];
                if (k + 1 < d) a.y = p[1];
                if (k + 2 < d) a.z = p[2];
                if (k + 3 < d) a.w = p[3];
            }
        }
        v[it] = a;
    }
}

__device__ __forceinline__ void store_slab(float *__restrict__ S, const float4 v[4])
{
    const int kq = (threadIdx.x & 7) * 4;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int r = (threadIdx.x >> 3) + 32 * it;
        *reinterpret_cast<float4 *>(S + r * LDS_STRIDE + kq) = v[it];
    }
}

// One 128 x 128 tile of query rows [q0 + 128 bx, ..) against database rows [j0 + 128 by, ..).
// TWO: two-level accumulation (needed once d exceeds KFLUSH); without it the kernel needs 64
// registers less and a third workgroup fits on a compute unit, which matters at small d, where
// the loads and the epilogue, not the matrix cores, set the pace.
template <bool TWO>
__global__ __launch_bounds__(256, TWO ? 2 : 3) void knn_tile_mfma(const float *__restrict__ X, int n, int d, int q0, int qend,
                                                     int j0, int jend, const float *__restrict__ norms,
                                                     const float *__restrict__ tau, int *__restrict__ cnt,
                                                     uint64_t *__restrict__ cand, int cap, int *__restrict__ ccount)
{
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *ccount = 0;   // for the compaction pass that follows
    __shared__ __align__(16) float As[TM * LDS_STRIDE];
    __shared__ __align__(16) float Bs[TN * LDS_STRIDE];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    const int qa = q0 + blockIdx.x * TM, ja = j0 + blockIdx.y * TN;
    const bool vec = (d & 3) == 0;
    // Two-level accumulation: the matrix cores sum KFLUSH columns into `part`, which is then added
    // to `acc` and cleared.  The rounding error of a dot product of length d drops from order d to
    // order KFLUSH + d / KFLUSH units in the last place, which is what lets a small candidate
    // margin certify rows at D in the thousands.
    floatx16 acc[TWO ? 2 : 1][TWO ? 2 : 1], part[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (TWO) acc[TWO ? a : 0][TWO ? b : 0][i] = 0.f;
                part[a][b][i] = 0.f;
            }
    float4 ra[4], rb[4];
    load_slab(X, d, qa, qend, 0, vec, ra);
    load_slab(X, d, ja, jend, 0, vec, rb);
    const int r32 = lane & 31, h = lane >> 5;
    for (int k0 = 0; k0 < d; k0 += BK) {
        __syncthreads();
        store_slab(As, ra);
        store_slab(Bs, rb);
        __syncthreads();
        if (k0 + BK < d) {
            load_slab(X, d, qa, qend, k0 + BK, vec, ra);
            load_slab(X, d, ja, jend, k0 + BK, vec, rb);
        }
        // each lane owns 16 of the slab's 32 columns (h selects the half); the same column
        // assignment is used for both operands, so the products pair up correctly.  The 16
        // columns are taken in two rounds of 8 to keep the fragment registers at 32.
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            float fa[2][8], fb[2][8];
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const float *pa = As + (wm * 64 + m * 32 + r32) * LDS_STRIDE + h * 16 + half * 8;
                const float *pb = Bs + (wn * 64 + m * 32 + r32) * LDS_STRIDE + h * 16 + half * 8;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    float4 va = *reinterpret_cast<const float4 *>(pa + 4 * q);
                    float4 vb = *reinterpret_cast<const float4 *>(pb + 4 * q);
                    fa[m][4 * q] = va.x; fa[m][4 * q + 1] = va.y; fa[m][4 * q + 2] = va.z; fa[m][4 * q + 3] = va.w;
                    fb[m][4 * q] = vb.x; fb[m][4 * q + 1] = vb.y; fb[m][4 * q + 2] = vb.z; fb[m][4 * q + 3] = vb.w;
                }
            }
#pragma unroll
            for (int s = 0; s < 8; ++s)
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        part[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a][s], fb[b][s], part[a][b], 0, 0, 0);
        }
        if (TWO && (((k0 / BK) % (KFLUSH / BK)) == (KFLUSH / BK) - 1 || k0 + BK >= d)) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
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
    __syncthreads();
    float *qn = As, *qt = As + TM;
    if (tid < TM) {
        const int q = qa + tid;
        qn[tid] = q < qend ? norms[q] : 0.f;
        qt[tid] = q < qend ? tau[q - q0] : -INFINITY;     // rows past the end accept nothing
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int j = ja + wn * 64 + b * 32 + r32;
        const float nj = j < jend ? norms[j] : 0.f;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int ql = wm * 64 + a * 32 + 8 * (i >> 2) + 4 * h + (i & 3);
                const int q = qa + ql;
                if (j < jend && j != q) {
                    const float dot = TWO ? acc[TWO ? a : 0][TWO ? b : 0][i] : part[a][b][i];
                    const float dist = (qn[ql] + nj) - 2.0f * dot;
                    if (dist < qt[ql]) {
                        const int pos = atomicAdd(&cnt[q - q0], 1);
                        if (pos < cap)
                            cand[(size_t)(q - q0) * cap + pos] = ((uint64_t)orderable(dist) << 32) | (uint32_t)j;
                    }
                }
            }
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
    if (!force && tau[row] < INFINITY && c < kp + COMPACT_SLACK && c + DBC <= cap) return;
    list[atomicAdd(count, 1)] = row;    // any order
}

__global__ __launch_bounds__(256) void knn_compact(float *__restrict__ tau, int *__restrict__ cnt,
                                                   uint64_t *__restrict__ cand, int cap, int kp, int rows,
                                                   const int *__restrict__ list, const int *__restrict__ count)
{
    __shared__ uint64_t s[SORT_CAP];
    const int m = min(*count, rows);
    for (int i = blockIdx.x; i < m; i += gridDim.x) {
    const int row = min(max(list[i], 0), rows - 1);
    int c = cnt[row];
    if (c > cap) c = cap;
    __syncthreads();                    // the previous row of this workgroup is out of s
    int size = 1;
    while (size < c) size <<= 1;
    uint64_t *buf = cand + (size_t)row * cap;
    for (int t = threadIdx.x; t < size; t += blockDim.x) s[t] = t < c ? buf[t] : ~0ull;
    __syncthreads();
    bitonic_sort(s, size);
    for (int t = threadIdx.x; t < kp; t += blockDim.x) buf[t] = s[t];
    if (threadIdx.x == 0) {
        cnt[row] = kp;
        tau[row] = unorderable((uint32_t)(s[kp - 1] >> 32));
    }
    }
}

// Exact distances of the candidates, final order, certificate.  One block per query row.
__global__ __launch_bounds__(256) void knn_rerank(const float *__restrict__ X, int n, int d, int q0, int rows, int k,
                                                  int kp, const float *__restrict__ norms, float norm_max,
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
    const int row = blockIdx.x;
    if (row >= rows) return;
    const int i = q0 + row;
    int c = cnt[row];
    if (c > kp) c = kp;
    const float *x = X + (size_t)i * d;
    for (int t = threadIdx.x; t < d; t += blockDim.x) xi[t] = x[t];
    __syncthreads();
    const uint64_t *buf = cand + (size_t)row * cap;
    const int w = threadIdx.x >> 6;
    for (int cidx = w; cidx < c; cidx += 4) {
        const int j = (int)(uint32_t)buf[cidx];
        const float *y = X + (size_t)j * d;
        double s = 0.0;
        for (int t = lane_id(); t < d; t += WAVE) { double df = (double)xi[t] - (double)y[t]; s += df * df; }
        s = wave_sum(s);
        if (lane_id() == 0) dd[cidx] = s;
    }
    __syncthreads();
    // rank by (distance, index): c <= 2048, plain counting rank is enough
    for (int a = threadIdx.x; a < c; a += blockDim.x) key[a] = orderable64(dd[a]);
    __syncthreads();
    for (int a = threadIdx.x; a < c; a += blockDim.x) {
        const uint64_t ka = key[a];
        const uint32_t ja = (uint32_t)buf[a];
        int r = 0;
        for (int b = 0; b < c; ++b) {
            const uint64_t kb = key[b];
            r += (kb < ka) || (kb == ka && (uint32_t)buf[b] < ja);
        }
        order[r] = a;
    }
    __syncthreads();
    for (int r = threadIdx.x; r < k && r < c; r += blockDim.x) {
        const int a = order[r];
        knn_idx[(size_t)i * k + r] = (int32_t)(uint32_t)buf[a];
        knn_d2[(size_t)i * k + r] = dd[a];
    }
    if (threadIdx.x == 0) {
        // pairs never kept had single-precision distance >= tau; the error of that distance is
        // at most E, so they are farther than the exact k-th candidate if tau - E > D_k
        bool ok = c >= k;
        if (ok && c < n - 1) {
            // error of the float distance: each product and each addition rounds once (2 KFLUSH per
            // partial sum), d / KFLUSH additions of partial sums, a few for norms and the final
            // combination; terms are bounded by (|q|^2 + |x|^2) / 2 in sum; the whole doubled for safety
            const double roundings = 2.0 * KFLUSH + (double)((d + KFLUSH - 1) / KFLUSH) + 16.0;
            const double E = roundings * 5.9604644775390625e-08 * ((double)norms[i] + (double)norm_max) * 2.0;
            const double Dk = dd[order[k - 1]];
            ok = (double)tau[row] - E > Dk;
        }
        if (!ok) fail_rows[atomicAdd(fail_count, 1)] = i;
    }
}

// ---- rows that failed the certificate: exact distances to every row, then selection
__global__ __launch_bounds__(256) void knn_exact_dists(const float *__restrict__ X, int n, int d, int i,
                                                       uint64_t *__restrict__ okey)
{
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= n) return;
    const float *x = X + (size_t)i * d, *y = X + (size_t)j * d;
    double s = 0.0;
    for (int t = lane_id(); t < d; t += WAVE) { double df = (double)x[t] - (double)y[t]; s += df * df; }
    s = wave_sum(s);
    if (lane_id() == 0) okey[j] = (j == i) ? ~0ull : orderable64(s);
}

// One block: 8 radix passes over the ordered 64-bit keys find the k-th smallest distance; then
// the keys below it and the lowest-index ties are put in (distance, index) order.
constexpr int TIE_CAP = 4096;

__device__ __forceinline__ double key_to_double(uint64_t v)
{
    const uint64_t u = (v & 0x8000000000000000ull) ? (v & 0x7FFFFFFFFFFFFFFFull) : ~v;
    return __longlong_as_double((long long)u);
}

__global__ __launch_bounds__(1024) void knn_exact_select(const uint64_t *__restrict__ okey, int n, int k, int i,
                                                         int32_t *__restrict__ knn_idx, double *__restrict__ knn_d2)
{
    __shared__ uint32_t hist[256];
    __shared__ uint64_t prefix_s;
    __shared__ int want_s, nsel, ntie;
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
            if (p < MAX_KP) { selk[p] = v; selj[p] = j; }
        } else if (v == prefix) {
            const int p = atomicAdd(&ntie, 1);
            if (p < TIE_CAP) tie[p] = (uint64_t)(uint32_t)j;
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
        knn_d2[(size_t)i * k + r] = key_to_double(ka);
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
            knn_d2[(size_t)i * k + below + t] = dk;
        }
    } else if (threadIdx.x == 0) {
        // more equidistant rows than the tie buffer holds: take them in index order, serially
        int out = below;
        for (int j = 0; j < n && out < k; ++j)
            if (okey[j] == prefix) { knn_idx[(size_t)i * k + out] = j; knn_d2[(size_t)i * k + out] = dk; ++out; }
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

__global__ __launch_bounds__(64) void perplexity_search(const double *__restrict__ d2, int n, int k, double target,
                                                        double tol, double *__restrict__ cond,
                                                        int *__restrict__ unconverged)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const double *dd = d2 + (size_t)i * k;
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
// slot of i in row j's neighbour list, or -1
__device__ __forceinline__ int find_in_row(const int32_t *__restrict__ idx, int k, int j, int i)
{
    const int32_t *r = idx + (size_t)j * k;
    for (int a = 0; a < k; ++a) if (r[a] == i) return a;
    return -1;
}

// extra[j] = number of rows i that list j while j does not list i
__global__ __launch_bounds__(256) void sym_count(const int32_t *__restrict__ idx, int n, int k, int *__restrict__ extra)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)n * k) return;
    const int i = (int)(e / k), j = idx[e];
    if (find_in_row(idx, k, j, i) < 0) atomicAdd(&extra[j], 1);
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
                                                int32_t *__restrict__ col, float *__restrict__ val)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)n * k) return;
    const int i = (int)(e / k), a = (int)(e % k), j = idx[e];
    const double pji = cond[e];
    const int slot = find_in_row(idx, k, j, i);
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
    const int row = blockIdx.x;
    if (row >= n) return;
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
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < m) out[i] = (float)in[i];
}

struct Layout {
    float *norms, *norm_max, *tau;
    int *cnt, *fail_count, *fail_rows, *extra, *cursor, *unconv;
    uint64_t *cand, *okey, *sort_scratch;
    int *clist, *ccount;     // rows of the current query block that need compaction, and how many
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
    (void)d;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += up(bytes); return (void *)p; };
    const int kp = margin_kp(n, k);
    const int cap = kp + COMPACT_SLACK + DBC;   // <= SORT_CAP because kp <= MAX_KP
    const size_t qb = (size_t)(n < QB ? n : QB);
    void *q;
    q = take(4 * (size_t)n); if (L) L->norms = (float *)q;
    q = take(4); if (L) L->norm_max = (float *)q;
    q = take(4 * qb); if (L) L->tau = (float *)q;
    q = take(4 * qb); if (L) L->cnt = (int *)q;
    q = take(4 * qb); if (L) L->clist = (int *)q;
    q = take(4); if (L) L->ccount = (int *)q;
    q = take(4); if (L) L->fail_count = (int *)q;
    q = take(4 * (size_t)n); if (L) L->fail_rows = (int *)q;
    q = take(4 * (size_t)n); if (L) L->extra = (int *)q;
    q = take(4 * (size_t)n); if (L) L->cursor = (int *)q;
    q = take(4); if (L) L->unconv = (int *)q;
    q = take(8 * qb * cap); if (L) L->cand = (uint64_t *)q;
    q = take(8 * (size_t)n); if (L) L->okey = (uint64_t *)q;
    q = take(8 * (size_t)2 * n * k); if (L) L->sort_scratch = (uint64_t *)q;
    q = take(4 * (size_t)n * k); if (L) L->knn_idx = (int32_t *)q;
    q = take(8 * (size_t)n * k); if (L) L->knn_d2 = (double *)q;
    q = take(8 * (size_t)n * k); if (L) L->cond = (double *)q;
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

extern "C" {

int tsne_build_P_workspace_bytes(int32_t n, int32_t d, int32_t k, size_t *bytes)
{
    if (!bytes || check_args(n, d, k) != TSNE_OK) return TSNE_EINVAL;
    *bytes = carve(nullptr, n, d, k, nullptr);
    return TSNE_OK;
}

#define HIPCHK(call)                                      \
    do {                                                  \
        hipError_t e_ = (call);                           \
        if (e_ != hipSuccess) {                           \
            fprintf(stderr, "tsne_build_P: %s failed: %s\n", #call, hipGetErrorString(e_)); \
            return TSNE_EHIP;                             \
        }                                                 \
    } while (0)

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

    hipLaunchKernelGGL(row_norms, dim3((n + 3) / 4), dim3(256), 0, s, d_X, n, d, L.norms);
    hipLaunchKernelGGL(max_norm_k, dim3(1), dim3(1024), 0, s, L.norms, n, L.norm_max);
    HIPCHK(hipMemsetAsync(L.fail_count, 0, 4, s));
    HIPCHK(hipMemsetAsync(L.unconv, 0, 4, s));
    HIPCHK(hipMemsetAsync(L.extra, 0, 4 * (size_t)n, s));
    float norm_max = 0.f;
    HIPCHK(hipMemcpyAsync(&norm_max, L.norm_max, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));

    const size_t rerank_smem = up((size_t)d * 4) + 8 * (size_t)MAX_KP;
    for (int q0 = 0; q0 < n; q0 += QB) {
        const int qend = q0 + QB < n ? q0 + QB : n, rows = qend - q0;
        hipLaunchKernelGGL(knn_reset, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, rows);
        for (int j0 = 0; j0 < n; j0 += DBC) {
            const int jend = j0 + DBC < n ? j0 + DBC : n;
            dim3 grid((rows + TM - 1) / TM, (jend - j0 + TN - 1) / TN);
            if (d > KFLUSH)
                hipLaunchKernelGGL(knn_tile_mfma<true>, grid, dim3(256), 0, s, d_X, n, d, q0, qend, j0, jend, L.norms,
                                   L.tau, L.cnt, L.cand, cap, L.ccount);
            else   // one flush at the end is the same sum
                hipLaunchKernelGGL(knn_tile_mfma<false>, grid, dim3(256), 0, s, d_X, n, d, q0, qend, j0, jend, L.norms,
                                   L.tau, L.cnt, L.cand, cap, L.ccount);
            hipLaunchKernelGGL(knn_compact_list, dim3((rows + 255) / 256), dim3(256), 0, s, L.tau, L.cnt, cap, kp, rows,
                               jend >= n ? 1 : 0, L.clist, L.ccount);
            hipLaunchKernelGGL(knn_compact, dim3(rows < 4096 ? rows : 4096), dim3(256), 0, s, L.tau, L.cnt, L.cand, cap,
                               kp, rows, L.clist, L.ccount);
        }
        hipLaunchKernelGGL(knn_rerank, dim3(rows), dim3(256), rerank_smem, s, d_X, n, d, q0, rows, k, kp, L.norms,
                           norm_max, L.tau, L.cnt, L.cand, cap, L.knn_idx, L.knn_d2, L.fail_count, L.fail_rows);
        HIPCHK(hipGetLastError());
    }
    int nfail = 0;
    HIPCHK(hipMemcpyAsync(&nfail, L.fail_count, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    if (nfail > 0) {
        int *rows_h = (int *)malloc(sizeof(int) * (size_t)nfail);
        if (!rows_h) return TSNE_ENOSPC;
        HIPCHK(hipMemcpyAsync(rows_h, L.fail_rows, 4 * (size_t)nfail, hipMemcpyDeviceToHost, s));
        HIPCHK(hipStreamSynchronize(s));
        for (int f = 0; f < nfail; ++f) {
            hipLaunchKernelGGL(knn_exact_dists, dim3((n + 3) / 4), dim3(256), 0, s, d_X, n, d, rows_h[f], L.okey);
            hipLaunchKernelGGL(knn_exact_select, dim3(1), dim3(1024), 0, s, L.okey, n, k, rows_h[f], L.knn_idx,
                               L.knn_d2);
        }
        free(rows_h);
        HIPCHK(hipGetLastError());
    }
    const size_t nk = (size_t)n * k;
    hipLaunchKernelGGL(perplexity_search, dim3((n + 63) / 64), dim3(64), 0, s, L.knn_d2, n, k, log((double)perplexity),
                       1e-10, L.cond, L.unconv);
    hipLaunchKernelGGL(sym_count, dim3((unsigned)((nk + 255) / 256)), dim3(256), 0, s, L.knn_idx, n, k, L.extra);
    hipLaunchKernelGGL(sym_scan, dim3(1), dim3(1024), 0, s, L.extra, n, k, d_row_ptr, L.cursor);
    int32_t total = 0;
    HIPCHK(hipMemcpyAsync(&total, d_row_ptr + n, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    if ((int64_t)total > cap_nnz) return TSNE_ENOSPC;
    hipLaunchKernelGGL(sym_fill, dim3((unsigned)((nk + 255) / 256)), dim3(256), 0, s, L.knn_idx, L.cond, n, k, d_row_ptr,
                       L.cursor, d_col, d_val);
    hipLaunchKernelGGL(sym_sort_rows, dim3(n), dim3(256), 0, s, d_row_ptr, n, d_col, d_val, L.sort_scratch);
    if (d_knn_idx) HIPCHK(hipMemcpyAsync(d_knn_idx, L.knn_idx, 4 * nk, hipMemcpyDeviceToDevice, s));
    if (d_knn_d2)
        hipLaunchKernelGGL(d2_to_float, dim3((unsigned)((nk + 255) / 256)), dim3(256), 0, s, L.knn_d2, d_knn_d2, nk);
    int unconv = 0;
    HIPCHK(hipMemcpyAsync(&unconv, L.unconv, 4, hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    HIPCHK(hipGetLastError());
    *nnz = total;
    if (n_unconverged) *n_unconverged = unconv;
    return TSNE_OK;
}

}  // extern "C"
