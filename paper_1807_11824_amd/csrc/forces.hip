// Attractive forces over the sparse P (Eq. (5), Alg. 1 lines 6-7 fused: P.Q is never stored),
// the update of the embedding (Alg. 1 line 8) and the exact-Z KL utility.
#include "tsne_internal.h"

#include <math.h>

// A_i = sum_j p_ij w_ij (y_i - y_j), w_ij = 1/(1+|y_i-y_j|^2).  LPR lanes share one CSR row:
// col/val are read as contiguous segments, y_j is an 8-byte gather, and the two partial sums
// are combined with xor-shuffles inside the LPR-lane group.  No atomics: the result is
// deterministic.
//
// Rows are visited in the order given by `order` (the spatial order of an earlier tree build):
// rows that are close in the embedding share most of their neighbours, so the y_j gathers of
// one workgroup and its neighbours on the chip keep hitting the same cache lines.  The result
// of a row does not depend on when it is computed.
// The kernel is bound by memory latency unless every lane keeps several independent loads in
// flight: each pass of a lane covers U entries (stride LPR), issues their y_j gathers together,
// then does the arithmetic.
template <int LPR, int U>
__global__ __launch_bounds__(256) void attract_csr(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col,
                                                   const float *__restrict__ val, const float2 *__restrict__ Y, int n,
                                                   const uint32_t *__restrict__ order, float2 *__restrict__ A)
{
    const int slot = (int)((blockIdx.x * 256u + threadIdx.x) / LPR);
    const int sub = (int)(threadIdx.x % LPR);
    float ax = 0.f, ay = 0.f;
    const int row = slot < n ? (int)min(order[slot], (uint32_t)n - 1u) : n;
    if (row < n) {
        const int s = row_ptr[row], e = row_ptr[row + 1];
        const float2 yi = Y[row];
        for (int j0 = s + sub; j0 < e; j0 += LPR * U) {
            int c[U];
            float v[U];
            float2 yj[U];
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const int j = j0 + q * LPR;
                const bool in = j < e;
                c[q] = in ? col[j] : row;     // padding: own point, weight 0
                v[q] = in ? val[j] : 0.f;
            }
#pragma unroll
            for (int q = 0; q < U; ++q) yj[q] = Y[min((uint32_t)c[q], (uint32_t)n - 1u)];
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const float dx = yi.x - yj[q].x, dy = yi.y - yj[q].y;
                const float w = __builtin_amdgcn_rcpf(fmaf(dy, dy, fmaf(dx, dx, 1.0f)));
                const float pw = v[q] * w;
                ax = fmaf(pw, dx, ax);
                ay = fmaf(pw, dy, ay);
            }
        }
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) {
        ax += __shfl_xor(ax, o, WAVE);
        ay += __shfl_xor(ay, o, WAVE);
    }
    if (row < n && sub == 0) A[row] = make_float2(ax, ay);
}

constexpr int AW_LPR = 16, AW_U = 4;

// ---- renumbered points: P is stored as a near part (a band around the diagonal) and a far part.
//
// attract_near streams the near part.  The grid is a fixed number of resident workgroups;
// workgroup b owns the contiguous rows [arow[b], arow[b + 1]) (equal shares of the entries) and
// moves through them ATTRACT_ROWS at a time.  Y of the band around the current rows lives in a
// ring in LDS that slides with the rows (only the points that enter are loaded), so every y_j
// gather is an LDS read -- the stored 16-bit column IS the byte offset into the ring -- and
// the only global loads of the inner loop are 16-byte pieces of the column and value streams
// (6 bytes per entry).  Four lanes share a row; a lane takes eight consecutive entries of each
// 32-entry chunk, and rows are stored padded to whole chunks so that no load needs a guard.
// Every group keeps AN_PD chunks in flight, requested unconditionally right after the stage's
// registers were used, so loads are issued long before they are needed and eight waves per
// compute unit keep HBM busy -- which leaves most of every compute unit to the tree walk that
// runs beside it (the kernel is held to 64 registers for the same reason).  Within one window
// step the rows are handed to the groups longest first through a counter in LDS, one row
// ahead; a row's sum does not depend on which group takes it or when.
constexpr int AN_THREADS = 512, AN_ROWS = ATTRACT_ROWS, AN_S = ATTRACT_RING, AN_LPR = 4, AN_CH = ATTRACT_CHUNK;
static_assert(AN_CH == 8 * AN_LPR, "a lane takes two quads of a chunk");
constexpr int AN_PD = 2, AN_GROUPS = AN_THREADS / AN_LPR;

// Shares of the rows for the k resident workgroups: equal work each, the work of rows [0, r)
// being their entries plus a fixed cost per row.
__global__ void attract_partition(const int32_t *__restrict__ rp_near, int n, int k, int32_t *__restrict__ arow)
{
    const int b = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (b > k) return;
    const int64_t total = (int64_t)rp_near[n] + 16ll * n;
    const int64_t target = total * b / k;
    int lo = 0, hi = n;   // smallest r with work(r) >= target
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)rp_near[mid] + 16ll * mid >= target) hi = mid; else lo = mid + 1;
    }
    arow[b] = b == k ? n : lo;
}

__global__ __attribute__((amdgpu_waves_per_eu(8))) __launch_bounds__(AN_THREADS) void
attract_near(const int32_t *__restrict__ rp, const uint4 *__restrict__ col8, const float4 *__restrict__ val4,
             const float2 *__restrict__ Y, int n, const int32_t *__restrict__ arow,
             const int32_t *__restrict__ rp_far, const float2 *__restrict__ Afar, float2 *__restrict__ A)
{
    __shared__ float2 ring[AN_S];
    __shared__ float2 aout[AN_ROWS];
    __shared__ int rps[AN_ROWS + 1];
    __shared__ int next_row;
    __shared__ int bucket[64];
    __shared__ uint16_t order[AN_ROWS];
    static_assert(AN_ROWS <= 65536, "rows per step");
    constexpr int KPT = (AN_ROWS + AN_THREADS - 1) / AN_THREADS;
    const int share = (int)blockIdx.x;
    const int rb = min(max(arow[share], 0), n), re = min(max(arow[share + 1], rb), n);
    if (rb >= re) return;
    const int tid = (int)threadIdx.x, sub = tid % AN_LPR, grp = tid / AN_LPR;
    const char *ringb = reinterpret_cast<const char *>(ring);
    for (int t = tid; t < 2 * ATTRACT_BAND; t += AN_THREADS) {
        const int i = rb - ATTRACT_BAND + t;
        if (i >= 0 && i < n) ring[(unsigned)i % AN_S] = Y[i];
    }
    int prev_r0 = 0, prev_rows = 0;
    for (int r0 = rb; r0 < re; r0 += AN_ROWS) {
        __syncthreads();   // the previous rows are finished: aout is complete, ring slots may be reused
        for (int t = tid; t < prev_rows; t += AN_THREADS) {   // near sum + far sum (where the row has a far part)
            const int r = prev_r0 + t;
            float2 a = aout[t];
            if (rp_far[r + 1] > rp_far[r]) { const float2 b = Afar[r]; a.x += b.x; a.y += b.y; }
            A[r] = a;
        }
        for (int t = tid; t < AN_ROWS; t += AN_THREADS) {
            const int i = r0 + ATTRACT_BAND + t;
            if (i < n) ring[(unsigned)i % AN_S] = Y[i];
        }
        const int rows = min(AN_ROWS, re - r0);
        for (int t = tid; t <= rows; t += AN_THREADS) rps[t] = rp[r0 + t];
        if (tid < 64) bucket[tid] = 0;
        if (tid == 0) next_row = 2 * AN_GROUPS;
        __syncthreads();
        // the rows are handed out longest first (counting sort by chunk count, 64 classes), so
        // that no group is left with a long row when the others have run out of work
        {
            int key[KPT], pos[KPT];
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const int t = tid + k * AN_THREADS;
                key[k] = 0; pos[k] = 0;
                if (t < rows) {
                    key[k] = 63 - min((rps[t + 1] - rps[t]) >> 5, 63);
                    pos[k] = atomicAdd(&bucket[key[k]], 1);
                }
            }
            __syncthreads();
            if (tid < 64) {
                int tot;
                const int ex = wave_excl_scan(bucket[tid], &tot);
                bucket[tid] = ex;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < KPT; ++k) {
                const int t = tid + k * AN_THREADS;
                if (t < rows) order[bucket[key[k]] + pos[k]] = (uint16_t)t;
            }
            __syncthreads();
        }
        const int slot0 = r0 % AN_S;     // ring slot of local row 0
        // cursor of this group: current row (local, -1 when there is none), next chunk, row end;
        // the row after it is fetched one row ahead so that the counter's latency stays hidden
        int crow = grp < rows ? (int)order[grp] : -1;
        int jb = crow >= 0 ? rps[crow] : 0, je = crow >= 0 ? rps[crow + 1] : 0;
        int nrow = grp + AN_GROUPS < rows ? (int)order[grp + AN_GROUPS] : -1;
        int njb = nrow >= 0 ? rps[nrow] : 0, nje = nrow >= 0 ? rps[nrow + 1] : 0;
        uint4 C[AN_PD];          // eight 16-bit ring offsets
        float4 V[AN_PD][2];
        int R[AN_PD];
        bool OK[AN_PD], FIN[AN_PD];
        float ax = 0.f, ay = 0.f;
        // request the cursor's next chunk into stage s and move the cursor (rows are whole
        // chunks; a lane takes entries 8 sub .. 8 sub + 7 of the chunk)
#define AN_ISSUE(s)                                                                      \
        {                                                                                \
            const int off_ = (jb >> 3) + sub;                                            \
            R[s] = crow;                                                                 \
            OK[s] = crow >= 0 && jb < je;                                                \
            FIN[s] = crow >= 0 && jb + AN_CH >= je;                                      \
            C[s] = col8[off_];                                                           \
            V[s][0] = val4[2 * off_];                                                    \
            V[s][1] = val4[2 * off_ + 1];                                                \
            if (__any(FIN[s])) {                                                         \
                int t_ = 0;                                                              \
                if (FIN[s] && sub == 0) t_ = atomicAdd(&next_row, 1);                    \
                t_ = first4(t_);                                                         \
                if (FIN[s]) {                                                            \
                    crow = nrow; jb = njb; je = nje;                                     \
                    nrow = t_ < rows ? (int)order[t_] : -1;                              \
                    njb = nrow >= 0 ? rps[nrow] : 0;                                     \
                    nje = nrow >= 0 ? rps[nrow + 1] : 0;                                 \
                } else if (crow >= 0) {                                                  \
                    jb += AN_CH;                                                         \
                }                                                                        \
            } else if (crow >= 0) {                                                      \
                jb += AN_CH;                                                             \
            }                                                                            \
        }
        // one interaction; o = byte offset of y_j in the ring
#define AN_ONE(o, p)                                                                     \
        {                                                                                \
            const float2 yj_ = *reinterpret_cast<const float2 *>(ringb + (o));   /* 8 (column mod ring) < 8 AN_S by construction */ \
            const float dx = yi.x - yj_.x, dy = yi.y - yj_.y;                            \
            const float w = __builtin_amdgcn_rcpf(fmaf(dy, dy, fmaf(dx, dx, 1.0f)));     \
            const float pw = (p) * w;                                                    \
            ax = fmaf(pw, dx, ax);                                                       \
            ay = fmaf(pw, dy, ay);                                                       \
        }
#pragma unroll
        for (int s = 0; s < AN_PD; ++s) AN_ISSUE(s)
        for (;;) {
            bool live = false;
#pragma unroll
            for (int s = 0; s < AN_PD; ++s) {
                const uint4 c = C[s];
                const float4 v0 = V[s][0], v1 = V[s][1];
                const int r = R[s];
                const bool ok = OK[s], fin = FIN[s];
                live |= r >= 0;
                if (ok) {
                    int sl = slot0 + r;
                    sl = sl >= AN_S ? sl - AN_S : sl;
                    const float2 yi = ring[sl];
                    AN_ONE(c.x & 0xFFFFu, v0.x) AN_ONE(c.x >> 16, v0.y) AN_ONE(c.y & 0xFFFFu, v0.z) AN_ONE(c.y >> 16, v0.w)
                    AN_ONE(c.z & 0xFFFFu, v1.x) AN_ONE(c.z >> 16, v1.y) AN_ONE(c.w & 0xFFFFu, v1.z) AN_ONE(c.w >> 16, v1.w)
                }
                if (__any(fin)) {
                    const float sx = sum4(ax), sy = sum4(ay);
                    if (fin) {
                        if (sub == 0) aout[r] = make_float2(sx, sy);
                        ax = ay = 0.f;
                    }
                }
                // refill the stage only now that its registers are free: requesting earlier
                // makes the compiler copy the arriving data at the loop end, which waits for it
                AN_ISSUE(s)
            }
            if (!__any(live)) break;
        }
#undef AN_ISSUE
#undef AN_ONE
        prev_r0 = r0;
        prev_rows = rows;
    }
    __syncthreads();
    for (int t = tid; t < prev_rows; t += AN_THREADS) {
        const int r = prev_r0 + t;
        float2 a = aout[t];
        if (rp_far[r + 1] > rp_far[r]) { const float2 b = Afar[r]; a.x += b.x; a.y += b.y; }
        A[r] = a;
    }
}

// The far part: sixteen lanes per listed row (the rows that have far entries, about one in seven
// on the benchmark workload), y_j gathered from memory.  Runs first, beside the tree build;
// attract_near adds the sums to its own.
__global__ __launch_bounds__(256) void attract_far(const int32_t *__restrict__ rp, const int32_t *__restrict__ col,
                                                   const float *__restrict__ val, const float2 *__restrict__ Y, int n,
                                                   const uint32_t *__restrict__ far_rows,
                                                   const uint32_t *__restrict__ far_count, float2 *__restrict__ Afar)
{
    const int sub = (int)(threadIdx.x % 16);
    const uint32_t m = min(*far_count, (uint32_t)n);
    const int far0 = rp[0];      // values sit behind the near part, columns start at 0
    for (uint32_t i = (blockIdx.x * 256u + threadIdx.x) / 16; i < m; i += gridDim.x * 16u) {
        const int row = (int)min(far_rows[i], (uint32_t)n - 1u);
        const int s = rp[row], e = rp[row + 1];
        const float2 yi = Y[row];
        float ax = 0.f, ay = 0.f;
        for (int j0 = s + sub; j0 < e; j0 += 16 * 4) {
            int c[4];
            float v[4];
            float2 yj[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = j0 + 16 * q;
                const bool in = j < e;
                c[q] = in ? col[j - far0] : row;
                v[q] = in ? val[j] : 0.f;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) yj[q] = Y[min((uint32_t)c[q], (uint32_t)n - 1u)];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float dx = yi.x - yj[q].x, dy = yi.y - yj[q].y;
                const float w = __builtin_amdgcn_rcpf(fmaf(dy, dy, fmaf(dx, dx, 1.0f)));
                const float pw = v[q] * w;
                ax = fmaf(pw, dx, ax);
                ay = fmaf(pw, dy, ay);
            }
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) {
            ax += __shfl_xor(ax, o, WAVE);
            ay += __shfl_xor(ay, o, WAVE);
        }
        if (sub == 0) Afar[row] = make_float2(ax, ay);
    }
}

// ---- the far part from its bucketed copy
// An entry of the far part costs attract_far a cache line for 8 bytes of Y.  When the far part is
// large (P without a band structure: one high-dimensional blob per cluster), the entries are taken
// tile by tile instead: a workgroup owns FT_ROWS rows and streams through their entries, which are
// stored by column tile of FT_COLS points, so that the positions y_j fetched around the same time
// share the 16 KB of one column tile and many are served by the first-level cache, which they have
// to themselves: the rows' own positions y_i sit in LDS beside the sums (24 bytes a row, 144 KB,
// one workgroup of 1024 lanes per compute unit).  Row sums are kept in fixed point -- 64-bit
// integers, so every addition is exact -- in LDS while the workgroup runs and added to a global
// array of doubles (whole numbers below 2^53) at its end (several workgroups may share a row tile,
// each taking a range of its entries): the result is exact for the terms as computed and does not
// depend on any order.
// The scale: a term is p w (y_i - y_j) with w <= 1, so a row sum is below
// (largest p) x (side of the tree's root square, which holds all of Y) x (longest far row) < 2^e; terms are multiplied by 2^(52 - e) and
// truncated to integers, which keeps every sum below 2^52.
__device__ __forceinline__ int ft_shift(const uint32_t *meta, const float4 *root)
{
    const float bound = __uint_as_float(meta[1]) * root->z * (float)meta[2];
    if (!(bound > 0.f) || !(bound < INFINITY)) return 0;
    int e;
    (void)frexpf(bound, &e);       // bound < 2^e
    return 52 - e;
}

constexpr int FT_THREADS = 1024;
constexpr int FT_UNROLL = 8;
constexpr size_t FT_LDS = (size_t)FT_ROWS * 24;     // two sums and the position of every row

typedef __attribute__((address_space(1))) double ft_glb_f64;

__global__ __launch_bounds__(FT_THREADS) void attract_far_tiled(const int32_t *__restrict__ ptr, const int32_t *__restrict__ tcol,
                                                                const uint16_t *__restrict__ trow,
                                                                const float *__restrict__ tval, const float2 *__restrict__ Y,
                                                                int n, int nct, const uint32_t *__restrict__ meta,
                                                                const float4 *__restrict__ root, double *__restrict__ gacc)
{
    if (!meta[0]) return;
    extern __shared__ __align__(16) unsigned char ft_smem[];
    // x sums, then y sums; row r of the tile at slot r ^ (r / 32 % 32): rows a fixed stride apart
    // (entries arrive roughly in row order) would otherwise meet in the same LDS banks
    long long *acc = reinterpret_cast<long long *>(ft_smem);      // integer sums: the terms are whole numbers
    float2 *yrow = reinterpret_cast<float2 *>(ft_smem + (size_t)FT_ROWS * 16);
    const uint32_t tid = threadIdx.x;
    const int rt = blockIdx.x, row0 = rt * FT_ROWS;
    // this workgroup's share of the row tile's entries
    const int t0 = ptr[(int64_t)rt * nct], t1 = ptr[(int64_t)(rt + 1) * nct];
    const int per = (int)(((int64_t)(t1 - t0) + gridDim.y - 1) / gridDim.y);
    const int s0 = t0 + (int)blockIdx.y * per, s1 = min(t1, s0 + per);
    if (s0 >= s1) return;                   // the same for every thread
    const int shift = ft_shift(meta, root);
    for (uint32_t t = tid; t < 2u * FT_ROWS; t += FT_THREADS) acc[t] = 0ll;
    for (uint32_t t = tid; t < (uint32_t)FT_ROWS; t += FT_THREADS) yrow[t] = Y[min((uint32_t)row0 + t, (uint32_t)n - 1u)];
    __syncthreads();
    // Entries past the end of the share are read as the share's last entry with weight 0 (they add 0).
    // The entries of the next trip are requested before the gathers of this one.
    const uint32_t last = (uint32_t)s1 - 1u;
    int32_t ncj[FT_UNROLL];
    uint16_t nrl[FT_UNROLL];
    float nv[FT_UNROLL];
    auto fetch = [&](uint32_t e0) {
#pragma unroll
        for (int u = 0; u < FT_UNROLL; ++u) {
            const uint32_t e = e0 + (uint32_t)u * FT_THREADS, ec = min(e, last);
            // (read once: kept out of the way of the lines of Y in the first-level cache)
            ncj[u] = __builtin_nontemporal_load(tcol + ec);
            nrl[u] = __builtin_nontemporal_load(trow + ec);
            nv[u] = __builtin_nontemporal_load(tval + ec);     // (nothing here uses what it loads)
        }
    };
    fetch((uint32_t)s0 + tid);
    for (uint32_t e0 = (uint32_t)s0 + tid; e0 <= last; e0 += FT_THREADS * FT_UNROLL) {
        uint32_t rl[FT_UNROLL];
        float v[FT_UNROLL];
        float2 yj[FT_UNROLL];
#pragma unroll
        for (int u = 0; u < FT_UNROLL; ++u) {
            rl[u] = min((uint32_t)nrl[u], (uint32_t)FT_ROWS - 1u);
            v[u] = e0 + (uint32_t)u * FT_THREADS <= last ? nv[u] : 0.f;
            yj[u] = Y[min((uint32_t)ncj[u], (uint32_t)n - 1u)];
        }
        // the memory counter is in order: all gathers go out before the next trip's entries are
        // requested, so that waiting for the gathers does not wait for those as well
        __builtin_amdgcn_sched_barrier(0);
        fetch(e0 + FT_THREADS * FT_UNROLL);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < FT_UNROLL; ++u) {
            const float2 yi = yrow[rl[u]];
            const float dx = yi.x - yj[u].x, dy = yi.y - yj[u].y;
            const float w = __builtin_amdgcn_rcpf(fmaf(dy, dy, fmaf(dx, dx, 1.0f)));
            const float pw = v[u] * w;
            const long long fx = (long long)ldexp((double)(pw * dx), shift), fy = (long long)ldexp((double)(pw * dy), shift);
            const uint32_t slot = rl[u] ^ ((rl[u] >> 5) & 31u);
            atomicAdd(reinterpret_cast<unsigned long long *>(acc + slot), (unsigned long long)fx);
            atomicAdd(reinterpret_cast<unsigned long long *>(acc + FT_ROWS + slot), (unsigned long long)fy);
        }
    }
    __syncthreads();
    for (uint32_t t = tid; t < 2u * FT_ROWS; t += FT_THREADS) {
        const uint32_t r = t / 2, slot = r ^ ((r >> 5) & 31u);
        const double a = (double)acc[(t & 1u) * FT_ROWS + slot];
        if (a != 0.0 && row0 + (int)r < n) {
            if (gridDim.y == 1) gacc[2 * (size_t)row0 + t] = a;      // the only workgroup of this row tile
            else (void)__builtin_amdgcn_global_atomic_fadd_f64((ft_glb_f64 *)(gacc + 2 * (size_t)row0 + t), a);
        }
    }
}

// fixed point -> float, and the accumulators back to zero for the next step
__global__ __launch_bounds__(256) void ft_finish_k(const uint32_t *__restrict__ far_rows, const uint32_t *__restrict__ far_count,
                                                   int n, const uint32_t *__restrict__ meta, const float4 *__restrict__ root,
                                                   double *__restrict__ gacc, float2 *__restrict__ Afar)
{
    if (!meta[0]) return;
    const uint32_t m = min(*far_count, (uint32_t)n);
    const int shift = ft_shift(meta, root);
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < m; i += gridDim.x * 256u) {
        const uint32_t row = min(far_rows[i], (uint32_t)n - 1u);
        const double ax = gacc[2 * (size_t)row], ay = gacc[2 * (size_t)row + 1];
        gacc[2 * (size_t)row] = 0.0;
        gacc[2 * (size_t)row + 1] = 0.0;
        Afar[row] = make_float2((float)ldexp(ax, -shift), (float)ldexp(ay, -shift));
    }
}

hipError_t attract_far_tiled_prepare()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&attract_far_tiled), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)FT_LDS);
}

constexpr int FAR_BLOCKS = 1024;
// number of resident workgroups of attract_near
static int attract_shares(const tsne_ctx *c)
{
    const int per_cu = c->p.attract_resident > 0 ? c->p.attract_resident : 1;
    const int tiles = (c->p.n + AN_ROWS - 1) / AN_ROWS;
    return max(1, min(min(per_cu * c->num_cu, ATTRACT_MAX_PARTS / 2), tiles));
}

// The far part from its tiles.  They need Y and the root square only: with two streams they are launched
// beside the tree build (whose kernels squeeze in as their workgroups end: 144 KB of LDS per workgroup
// leave no room on a compute unit for anything else), so that the step is the far part plus the walk and
// not tree build plus walk plus far part; with one stream, or when root, keys and order come out of a
// single launch, behind the walk.
static void launch_far_tiles(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n;
    // enough workgroups to fill the chip: a row tile's entries are shared out when there are few row tiles
    const int nrt = (n + FT_ROWS - 1) / FT_ROWS;
    // ... but no more than leave a workgroup some 64k entries: each one clears, fills and adds up to 6144 rows' sums
    int split = max(1, min(64, (8 * c->num_cu + nrt - 1) / nrt));
    if (c->ft_far_entries > 0) {
        const int64_t by_size = c->ft_far_entries / ((int64_t)nrt * 65536);
        if (by_size < split) split = by_size < 1 ? 1 : (int)by_size;
    }
    hipLaunchKernelGGL(attract_far_tiled, dim3((unsigned)nrt, (unsigned)split), dim3(FT_THREADS), FT_LDS, s, c->ft_ptr,
                       c->ft_col, c->ft_row, c->ft_val, c->Yi, n, c->ft_nct, c->ft_meta, c->root, c->ft_acc);
    hipLaunchKernelGGL(ft_finish_k, dim3((unsigned)min((n + 255) / 256, 1024)), dim3(256), 0, s, c->far_rows, c->far_count, n,
                       c->ft_meta, c->root, c->ft_acc, c->Afar);
}

// The far part of the renumbered P when it is summed row by row (also shares the rows of the
// streaming part out, once per P).
hipError_t launch_attract_far(tsne_ctx *c, hipStream_t s, bool tiles)
{
    const int n = c->p.n;
    if (!(c->reorder_on && !c->identity)) return hipSuccess;
    if (!c->arow_valid) {   // P changed since the rows were shared out
        const int k = attract_shares(c);
        hipLaunchKernelGGL(attract_partition, dim3((k + 256) / 256), dim3(256), 0, s, c->rp_near, n, k, c->arow);
        c->arow_valid = 1;
    }
    if (c->ft_active && tiles) launch_far_tiles(c, s);
    if (!c->ft_active)
        hipLaunchKernelGGL(attract_far, dim3((unsigned)min((n + 15) / 16, FAR_BLOCKS)), dim3(256), 0, s, c->rp_far, c->col_far,
                           c->val_s, c->Yi, n, c->far_rows, c->far_count, c->Afar);
    return hipGetLastError();
}

hipError_t launch_attract_main(tsne_ctx *c, hipStream_t s, bool tiles)
{
    const int n = c->p.n;
    if (c->reorder_on && !c->identity) {
        if (c->ft_active && tiles) launch_far_tiles(c, s);
        hipLaunchKernelGGL(attract_near, dim3(attract_shares(c)), dim3(AN_THREADS), 0, s, c->rp_near,
                           (const uint4 *)c->col_near, (const float4 *)c->val_s, c->Yi, n, c->arow, c->rp_far, c->Afar, c->A);
    } else {
        const unsigned blocks = (unsigned)(((int64_t)n * AW_LPR + 255) / 256);
        hipLaunchKernelGGL((attract_csr<AW_LPR, AW_U>), dim3(blocks), dim3(256), 0, s, c->user_row_ptr, c->user_col,
                           c->user_val, c->Yi, n, c->row_order, c->A);
    }
    return hipGetLastError();
}

// Alg. 1 line 8.  grad = 4 (alpha A - R / Z) (Eq. (7)); per coordinate the gain grows by
// gain_inc when gradient and velocity differ in sign (sign in {-1,0,+1}) and is multiplied by
// gain_dec otherwise, floored at gain_min; velocity = momentum velocity - lr gain grad;
// y += velocity.
__device__ __forceinline__ int sign3(float v) { return v > 0.f ? 1 : (v < 0.f ? -1 : 0); }

// With `part` set the kernel also leaves what the next iteration starts from: the new point in
// slot order (Yi) and the workgroup's bounding box, so that a run of several iterations neither
// gathers Y again nor makes a separate pass for the box (Sec. III-C step 1).
__global__ __launch_bounds__(256) void update_k(float2 *__restrict__ Y, const uint32_t *__restrict__ orig, float2 *Yi,
                                                float2 *__restrict__ uY, float2 *__restrict__ gains,
                                                const float2 *__restrict__ A, const float2 *__restrict__ R,
                                                const double *__restrict__ Z, int n, float alpha, float momentum,
                                                float lr, float gain_inc, float gain_dec, float gain_min,
                                                float4 *__restrict__ part, uint32_t *status, int write_user)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = s < n;
    // Once the device has reported trouble (a non-finite coordinate, a tree or a walk that did not
    // fit) the forces of this step are not to be trusted: embedding and optimiser state stay as they are.
    const bool frozen = *status != 0u;
    float2 y = make_float2(0.f, 0.f);
    if (live) y = Yi[s];
    if (live && !frozen) {
        const double Zd = *Z;
        const float invZ = Zd > 0.0 ? (float)(1.0 / Zd) : 0.f;    // a single point has no pairs: Z = 0, R = 0
        const float2 a = A[s], r = R[s];
        float2 g = gains[s], u = uY[s];
        const float gx = 4.0f * (alpha * a.x - r.x * invZ), gy = 4.0f * (alpha * a.y - r.y * invZ);
        g.x = (sign3(gx) != sign3(u.x)) ? g.x + gain_inc : g.x * gain_dec;
        g.y = (sign3(gy) != sign3(u.y)) ? g.y + gain_inc : g.y * gain_dec;
        g.x = fmaxf(g.x, gain_min); g.y = fmaxf(g.y, gain_min);
        u.x = momentum * u.x - lr * g.x * gx;
        u.y = momentum * u.y - lr * g.y * gy;
        gains[s] = g;
        uY[s] = u;
        y.x += u.x; y.y += u.y;
        // (inside a run of several iterations only the last one has to reach the caller's array)
        if (write_user) Y[min(orig[s], (uint32_t)n - 1u)] = y;
    }
    if (!part) return;
    if (live) Yi[s] = y;
    const bool bad = live && !(isfinite(y.x) && isfinite(y.y));
    float mnx = wave_min(live ? y.x : INFINITY), mny = wave_min(live ? y.y : INFINITY);
    float mxx = wave_max(live ? y.x : -INFINITY), mxy = wave_max(live ? y.y : -INFINITY);
    __shared__ float4 smn[4], smx[4];
    const int w = threadIdx.x >> 6;
    if (lane_id() == 0) { smn[w] = make_float4(mnx, mny, 0, 0); smx[w] = make_float4(mxx, mxy, 0, 0); }
    if (__any(bad) && lane_id() == 0) atomicOr(status, TSNE_STATUS_NONFINITE);
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < 4; ++k) {
            mnx = fminf(mnx, smn[k].x); mny = fminf(mny, smn[k].y);
            mxx = fmaxf(mxx, smx[k].x); mxy = fmaxf(mxy, smx[k].y);
        }
        part[2 * blockIdx.x] = make_float4(mnx, mny, 0, 0);
        part[2 * blockIdx.x + 1] = make_float4(mxx, mxy, 0, 0);
    }
}

hipError_t launch_update(tsne_ctx *c, float *d_Y, float alpha, float momentum, int keep, int write_user, hipStream_t s)
{
    const int n = c->p.n, nb = (n + 255) / 256;
    hipLaunchKernelGGL(update_k, dim3(nb), dim3(256), 0, s, (float2 *)d_Y, c->orig[c->cur_state], c->Yi,
                       c->uYb[c->cur_state], c->gainsb[c->cur_state], c->A, c->R, c->Z, n, alpha, momentum, c->p.lr,
                       c->p.gain_inc, c->p.gain_dec, c->p.gain_min, keep ? c->bbox_part : (float4 *)nullptr, c->status,
                       write_user);
    if (keep) c->bbox_nparts = nb;
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_state_k(float *__restrict__ uY, float *__restrict__ gains, int n2)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < n2) { uY[c] = 0.f; gains[c] = 1.f; }
}

__global__ __launch_bounds__(256) void iota_k(uint32_t *__restrict__ a, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) a[i] = (uint32_t)i;
}

hipError_t launch_iota(uint32_t *a, int n, hipStream_t s)
{
    hipLaunchKernelGGL(iota_k, dim3((n + 255) / 256), dim3(256), 0, s, a, n);
    return hipGetLastError();
}

hipError_t launch_fill_state(tsne_ctx *c, hipStream_t s)
{
    const int n2 = 2 * c->p.n;
    hipLaunchKernelGGL(fill_state_k, dim3((n2 + 255) / 256), dim3(256), 0, s, (float *)c->uYb[c->cur_state],
                       (float *)c->gainsb[c->cur_state], n2);
    return hipGetLastError();
}

// ------------------------------------------------------------------ KL with exact Z (harness utility)
// Z of Eq. (4) over all ordered pairs: tile j through LDS, accumulate in double per block.
constexpr int KL_BLOCKS = 1024;

__global__ __launch_bounds__(256) void exact_z_k(const float2 *__restrict__ Y, int n, double *__restrict__ part)
{
    __shared__ float2 tile[256];
    __shared__ double ws[4];
    double acc = 0.0;
    for (int i0 = blockIdx.x * 256; i0 < n; i0 += gridDim.x * 256) {
        const int i = i0 + threadIdx.x;
        const float2 yi = Y[i < n ? i : 0];
        float z = 0.f;
        for (int j0 = 0; j0 < n; j0 += 256) {
            __syncthreads();
            const int j = j0 + threadIdx.x;
            tile[threadIdx.x] = j < n ? Y[j] : make_float2(INFINITY, INFINITY);   // w = 0
            __syncthreads();
            float zt = 0.f;
#pragma unroll 8
            for (int t = 0; t < 256; ++t) {
                const float dx = yi.x - tile[t].x, dy = yi.y - tile[t].y;
                zt += 1.0f / (fmaf(dy, dy, fmaf(dx, dx, 1.0f)));
            }
            z += zt;
        }
        if (i < n) acc += (double)z - 1.0;   // the j = i term contributed exactly 1
    }
    acc = wave_sum(acc);
    if (lane_id() == 0) ws[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = ws[0] + ws[1] + ws[2] + ws[3];
}

// sum over stored entries of p ln(p (1+d^2)); rows over a grid-stride loop
__global__ __launch_bounds__(256) void kl_terms_k(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col,
                                                  const float *__restrict__ val, const float2 *__restrict__ Y, int n,
                                                  double *__restrict__ part_t, double *__restrict__ part_p)
{
    __shared__ double ws[4], wp[4];
    double t = 0.0, ps = 0.0;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) {
        const float2 yi = Y[i];
        for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            const double pv = (double)val[e];
            if (!(pv > 0.0)) continue;
            const float2 yj = Y[col[e]];
            const double dx = (double)yi.x - (double)yj.x, dy = (double)yi.y - (double)yj.y;
            t += pv * log(pv * (1.0 + dx * dx + dy * dy));
            ps += pv;
        }
    }
    t = wave_sum(t); ps = wave_sum(ps);
    if (lane_id() == 0) { ws[threadIdx.x >> 6] = t; wp[threadIdx.x >> 6] = ps; }
    __syncthreads();
    if (threadIdx.x == 0) {
        part_t[blockIdx.x] = ws[0] + ws[1] + ws[2] + ws[3];
        part_p[blockIdx.x] = wp[0] + wp[1] + wp[2] + wp[3];
    }
}

// KL = sum p ln(p/q) = sum p ln(p (1+d^2)) + ln Z sum p
__global__ void kl_final_k(double *__restrict__ part, int nb)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double Z = 0.0, t = 0.0, ps = 0.0;
    for (int i = 0; i < nb; ++i) { Z += part[i]; t += part[nb + i]; ps += part[2 * nb + i]; }
    part[0] = t + log(Z) * ps;
    part[1] = Z;
}

__global__ void kl_copy_out_k(const double *__restrict__ part, double *__restrict__ out)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { out[0] = part[0]; out[1] = part[1]; }
}

hipError_t launch_kl(tsne_ctx *c, const float *d_Y, hipStream_t s)
{
    const int n = c->p.n;
    const float2 *Y = (const float2 *)d_Y;
    hipLaunchKernelGGL(exact_z_k, dim3(KL_BLOCKS), dim3(256), 0, s, Y, n, c->kl_part);
    hipLaunchKernelGGL(kl_terms_k, dim3(KL_BLOCKS), dim3(256), 0, s, c->user_row_ptr, c->user_col, c->user_val, Y, n,
                       c->kl_part + KL_BLOCKS, c->kl_part + 2 * KL_BLOCKS);
    hipLaunchKernelGGL(kl_final_k, dim3(1), dim3(64), 0, s, c->kl_part, KL_BLOCKS);
    return hipGetLastError();
}

// ------------------------------------------------------------------ the same utility for callers that cannot allocate
// tsne_kl_static: the three kernels above with their partial sums in a file-scope device array
// instead of a context's workspace, so that no context (and no allocation of any kind) is needed.
// Every GPU holds its own copy of the array at its own address, looked up once per device.
static __device__ __align__(256) double scratch[3 * KL_BLOCKS];
constexpr int KL_STATIC_MAX_DEVICES = 64;
static double *scratch_ptr[KL_STATIC_MAX_DEVICES];     // device address of `scratch`, by device ordinal

extern "C" int tsne_kl_static(const float *d_Y, int32_t n, const int32_t *d_row_ptr, const int32_t *d_col,
                              const float *d_val, double *d_out, void *stream)
{
    if (!d_Y || !d_row_ptr || !d_out || n < 1 || n > TSNE_KL_STATIC_MAX_N) return TSNE_EINVAL;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return TSNE_EHIP;
    if (dev < 0 || dev >= KL_STATIC_MAX_DEVICES) return TSNE_EINVAL;
    if (!scratch_ptr[dev]) {
        double *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TSNE_EHIP;
        scratch_ptr[dev] = ptr;
    }
    double *part = scratch_ptr[dev];
    hipStream_t s = (hipStream_t)stream;
    const float2 *Y = (const float2 *)d_Y;
    // every launch writes all of its KL_BLOCKS partial sums, so nothing of an earlier call is read
    hipLaunchKernelGGL(exact_z_k, dim3(KL_BLOCKS), dim3(256), 0, s, Y, n, part);
    hipLaunchKernelGGL(kl_terms_k, dim3(KL_BLOCKS), dim3(256), 0, s, d_row_ptr, d_col, d_val, Y, n, part + KL_BLOCKS,
                       part + 2 * KL_BLOCKS);
    hipLaunchKernelGGL(kl_final_k, dim3(1), dim3(64), 0, s, part, KL_BLOCKS);
    hipLaunchKernelGGL(kl_copy_out_k, dim3(1), dim3(64), 0, s, part, d_out);
    return hipGetLastError() == hipSuccess ? TSNE_OK : TSNE_EHIP;
}
