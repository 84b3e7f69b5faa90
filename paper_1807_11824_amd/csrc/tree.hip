// Sec. III-C steps 1-4 of the paper on gfx950: bounding box, grid keys, spatial sort,
// quad tree and cell summaries.  Nothing here walks pointers or inserts points one by one:
// the tree is read off the sorted keys.
//
//   bbox_partial / bbox_final   step 1   min/max reduction -> root square (power-of-two side)
//   morton_encode               step 2a  16-bit grid coordinates, bit-interleaved key
//   radix_hist / _scan / _scatter  step 4  stable LSD radix sort of (key, index), 8 bits a pass
//   small_root_keys_sort        steps 1, 2a, 4 in one launch of one workgroup, for few points
//   gather_levels               step 2b  which cells start at each sorted position
//   scan_partials / downsweep   step 3   prefix sums: cell numbering and running coordinate sums
//   write_cells                 steps 2c+3  cell records: members, count, centre of mass, children
//
// A cell at depth t is the run of sorted positions sharing the top 2t key bits.  A position p
// opens cells at depths tmin(p).. where tmin is fixed by the first digit in which key[p] differs
// from key[p-1]; the chain stops at the first depth whose parent holds <= leaf_cap points.
// Numbering cells by (position, depth) is exactly depth-first pre-order, so one scalar prefix
// sum over "cells opened at p" numbers the whole tree, and the centre of mass of any cell is a
// difference of two entries of the double-precision running sum of the sorted coordinates.
#include "tsne_internal.h"

#include <math.h>

// ------------------------------------------------------------------ bounding box
// Also brings the caller's Y (original point order) into the library's slot order:
// Yi[s] = Y[orig[s]].
__global__ __launch_bounds__(256) void bbox_partial(const float2 *__restrict__ Y, const uint32_t *__restrict__ orig,
                                                    float2 *__restrict__ Yi, int n, float4 *__restrict__ part,
                                                    uint32_t *status)
{
    float mnx = INFINITY, mny = INFINITY, mxx = -INFINITY, mxy = -INFINITY;
    bool bad = false;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        float2 y = Y[min(orig[i], (uint32_t)n - 1u)];
        Yi[i] = y;
        bad |= !(isfinite(y.x) && isfinite(y.y));
        mnx = fminf(mnx, y.x); mxx = fmaxf(mxx, y.x);
        mny = fminf(mny, y.y); mxy = fmaxf(mxy, y.y);
    }
    mnx = wave_min(mnx); mny = wave_min(mny); mxx = wave_max(mxx); mxy = wave_max(mxy);
    __shared__ float4 smn[4], smx[4];
    int w = threadIdx.x >> 6;
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

// Root square: lower corner (min x, min y); side = smallest power of two >= the larger extent,
// at least 2^-40; scale S = 2^bits / side (an exact power of two).
__device__ __forceinline__ float4 root_square(float mnx, float mny, float mxx, float mxy, int bits, uint32_t *status)
{
    float ex = mxx - mnx, ey = mxy - mny;
    float e = fmaxf(ex, ey);
    float W = ldexpf(1.0f, -40);
    if (!isfinite(e) || !isfinite(mnx) || !isfinite(mny)) {
        atomicOr(status, TSNE_STATUS_NONFINITE);
        mnx = 0.0f; mny = 0.0f; W = 1.0f;
    } else if (e > W) {
        int ex2;
        float m = frexpf(e, &ex2);          // e = m 2^ex2, m in [0.5, 1)
        W = (m == 0.5f) ? e : ldexpf(1.0f, ex2);
    }
    float S = ldexpf(1.0f, bits) / W;
    return make_float4(mnx, mny, W, S);
}

__global__ __launch_bounds__(1024) void bbox_final(const float4 *__restrict__ part, int nparts, int bits,
                                                   float4 *__restrict__ root, uint32_t *status)
{
    float mnx = INFINITY, mny = INFINITY, mxx = -INFINITY, mxy = -INFINITY;
    for (int i = threadIdx.x; i < nparts; i += blockDim.x) {
        float4 a = part[2 * i], b = part[2 * i + 1];
        mnx = fminf(mnx, a.x); mny = fminf(mny, a.y);
        mxx = fmaxf(mxx, b.x); mxy = fmaxf(mxy, b.y);
    }
    mnx = wave_min(mnx); mny = wave_min(mny); mxx = wave_max(mxx); mxy = wave_max(mxy);
    __shared__ float4 smn[16], smx[16];
    const int w = threadIdx.x >> 6, nw = (int)(blockDim.x >> 6);
    if (lane_id() == 0) { smn[w] = make_float4(mnx, mny, 0, 0); smx[w] = make_float4(mxx, mxy, 0, 0); }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < nw; ++k) {
            mnx = fminf(mnx, smn[k].x); mny = fminf(mny, smn[k].y);
            mxx = fmaxf(mxx, smx[k].x); mxy = fmaxf(mxy, smx[k].y);
        }
        *root = root_square(mnx, mny, mxx, mxy, bits, status);
    }
}

// ------------------------------------------------------------------ grid keys
__device__ __forceinline__ uint32_t spread16(uint32_t v)
{
    v &= 0xFFFFu;
    v = (v | (v << 8)) & 0x00FF00FFu;
    v = (v | (v << 4)) & 0x0F0F0F0Fu;
    v = (v | (v << 2)) & 0x33333333u;
    v = (v | (v << 1)) & 0x55555555u;
    return v;
}

// One rounding per operation: the subtraction rounds, the product with a power of two is exact.
__device__ __forceinline__ uint32_t grid_coord(float v, float origin, float S, uint32_t qmax)
{
#pragma clang fp contract(off)
    float r = v - origin;
    float s = r * S;
    float f = floorf(s);
    return f >= (float)qmax ? qmax : (f > 0.0f ? (uint32_t)f : 0u);
}

__global__ __launch_bounds__(256) void morton_encode(const float2 *__restrict__ Y, int n,
                                                     const float4 *__restrict__ root, int bits,
                                                     uint32_t *__restrict__ keys_orig,
                                                     uint32_t *__restrict__ keys, uint32_t *__restrict__ idx)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float4 r = *root;
    float2 y = Y[i];
    uint32_t qmax = (1u << bits) - 1u;
    uint32_t qx = grid_coord(y.x, r.x, r.w, qmax);
    uint32_t qy = grid_coord(y.y, r.y, r.w, qmax);
    uint32_t key = spread16(qx) | (spread16(qy) << 1);
    keys_orig[i] = key;
    keys[i] = key;
    idx[i] = (uint32_t)i;
}

// ------------------------------------------------------------------ few points: one workgroup does it all
// Root square, keys and the sort of (key, index) in one launch, for n <= SMALL_SORT_MAX: the pairs
// sit in LDS as key * 2^32 + index (all different, so any sorting network gives the order of a
// stable sort by key), padded with all-ones to m, the power of two >= n.  Same root, same keys
// and same order as bbox_final + morton_encode + the radix passes.
//
// The network is the bitonic one.  A thread holds E = 2^LOGE pairs that differ in LOGE
// neighbouring index bits, so one trip through LDS serves LOGE exchange distances; one padding
// slot after every eight keeps the lanes of a wave on different banks whichever bits they are.
__device__ __forceinline__ int small_sort_slot(int i) { return i + (i >> 3); }

template <int LOGE>
__device__ __forceinline__ void bitonic_trip(unsigned long long *pairs, int t, int b_lo, int nsteps, int k)
{
    constexpr int E = 1 << LOGE;
    const int base = ((t >> b_lo) << (b_lo + LOGE)) | (t & ((1 << b_lo) - 1));
    unsigned long long v[E];
#pragma unroll
    for (int e = 0; e < E; ++e) v[e] = pairs[small_sort_slot(base | (e << b_lo))];
    // direction of the run of length k a pair belongs to: one per thread unless k's bit is among the E's
    if ((k >> (b_lo + LOGE)) != 0) {
        const bool up = (base & k) == 0;
#pragma unroll
        for (int c = LOGE - 1; c >= 0; --c) {
            if (c < nsteps) {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    if (e & (1 << c)) continue;
                    unsigned long long a = v[e], b = v[e | (1 << c)];
                    const bool sw = (a > b) == up;
                    v[e] = sw ? b : a;
                    v[e | (1 << c)] = sw ? a : b;
                }
            }
        }
    } else {
#pragma unroll
        for (int c = LOGE - 1; c >= 0; --c) {
            if (c < nsteps) {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    if (e & (1 << c)) continue;
                    const bool up = ((e << b_lo) & k) == 0;
                    unsigned long long a = v[e], b = v[e | (1 << c)];
                    const bool sw = (a > b) == up;
                    v[e] = sw ? b : a;
                    v[e | (1 << c)] = sw ? a : b;
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < E; ++e) pairs[small_sort_slot(base | (e << b_lo))] = v[e];
}

// blockDim.x = m >> LOGE
template <int LOGE>
__global__ __launch_bounds__(1024) void small_root_keys_sort(const float2 *__restrict__ Y, int n, int m,
                                                             const float4 *__restrict__ part, int nparts, int bits,
                                                             float4 *__restrict__ root, uint32_t *__restrict__ keys_orig,
                                                             uint32_t *__restrict__ keys_out,
                                                             uint32_t *__restrict__ idx_out, uint32_t *status)
{
    extern __shared__ unsigned long long pairs[];
    __shared__ float4 smn[16], smx[16];
    __shared__ float4 sroot;
    const int tid = threadIdx.x, nthr = blockDim.x;
    {
        float mnx = INFINITY, mny = INFINITY, mxx = -INFINITY, mxy = -INFINITY;
        for (int i = tid; i < nparts; i += nthr) {
            float4 a = part[2 * i], b = part[2 * i + 1];
            mnx = fminf(mnx, a.x); mny = fminf(mny, a.y);
            mxx = fmaxf(mxx, b.x); mxy = fmaxf(mxy, b.y);
        }
        mnx = wave_min(mnx); mny = wave_min(mny); mxx = wave_max(mxx); mxy = wave_max(mxy);
        const int w = tid >> 6, nw = nthr >> 6;
        if (lane_id() == 0) { smn[w] = make_float4(mnx, mny, 0, 0); smx[w] = make_float4(mxx, mxy, 0, 0); }
        __syncthreads();
        if (tid == 0) {
            for (int k = 1; k < nw; ++k) {
                mnx = fminf(mnx, smn[k].x); mny = fminf(mny, smn[k].y);
                mxx = fmaxf(mxx, smx[k].x); mxy = fmaxf(mxy, smx[k].y);
            }
            float4 r = root_square(mnx, mny, mxx, mxy, bits, status);
            sroot = r;
            *root = r;
        }
        __syncthreads();
    }
    const float4 r = sroot;
    const uint32_t qmax = (1u << bits) - 1u;
    for (int i = tid; i < m; i += nthr) {
        unsigned long long v = ~0ull;
        if (i < n) {
            float2 y = Y[i];
            uint32_t qx = grid_coord(y.x, r.x, r.w, qmax);
            uint32_t qy = grid_coord(y.y, r.y, r.w, qmax);
            uint32_t key = spread16(qx) | (spread16(qy) << 1);
            keys_orig[i] = key;
            v = ((unsigned long long)key << 32) | (uint32_t)i;
        }
        pairs[small_sort_slot(i)] = v;
    }
    __syncthreads();
    // stage s makes sorted runs of length 2^s out of pairs of runs of opposite direction: exchanges at
    // distances 2^(s-1) .. 1, taken LOGE at a time from the top
    for (int st = 1; (1 << st) <= m; ++st) {
        for (int rem = st; rem > 0;) {
            const int ns = rem < LOGE ? rem : LOGE;
            bitonic_trip<LOGE>(pairs, tid, rem - ns, ns, 1 << st);
            rem -= ns;
            __syncthreads();
        }
    }
    for (int i = tid; i < n; i += nthr) {
        unsigned long long v = pairs[small_sort_slot(i)];
        keys_out[i] = (uint32_t)(v >> 32);
        idx_out[i] = (uint32_t)v;
    }
}

static size_t small_sort_lds(int m) { return 8 * (size_t)(m + (m >> 3)); }

hipError_t small_sort_prepare()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&small_root_keys_sort<3>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)small_sort_lds(SMALL_SORT_MAX));
}

// ------------------------------------------------------------------ radix sort (stable, LSD, 8 bits)
// hist layout: hist[digit * nblk + block].
__global__ __launch_bounds__(SORT_THREADS) void radix_hist(const uint32_t *__restrict__ keys, int n, int shift,
                                                           uint32_t *__restrict__ hist, int nblk)
{
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    int base = blockIdx.x * SORT_TILE;
#pragma unroll
    for (int r = 0; r < SORT_ITEMS; ++r) {
        int e = base + r * SORT_THREADS + threadIdx.x;
        if (e < n) atomicAdd(&h[(keys[e] >> shift) & 0xFFu], 1u);
    }
    __syncthreads();
    hist[threadIdx.x * nblk + blockIdx.x] = h[threadIdx.x];
}

// Block d turns hist[d][0..nblk) into its exclusive prefix and stores the digit total.
__global__ __launch_bounds__(256) void radix_scan(uint32_t *__restrict__ hist, int nblk, uint32_t *__restrict__ dtot)
{
    __shared__ uint32_t wsum[4];
    uint32_t *row = hist + (size_t)blockIdx.x * nblk;
    uint32_t carry = 0;
    int w = threadIdx.x >> 6;
    for (int b0 = 0; b0 < nblk; b0 += 256) {
        int b = b0 + threadIdx.x;
        int v = b < nblk ? (int)row[b] : 0;
        int tot;
        int ex = wave_excl_scan(v, &tot);
        if (lane_id() == 0) wsum[w] = (uint32_t)tot;
        __syncthreads();
        uint32_t wbase = 0, all = 0;
        for (int k = 0; k < 4; ++k) { if (k < w) wbase += wsum[k]; all += wsum[k]; }
        if (b < nblk) row[b] = carry + wbase + (uint32_t)ex;
        carry += all;
        __syncthreads();
    }
    if (threadIdx.x == 0) dtot[blockIdx.x] = carry;
}

__global__ __launch_bounds__(SORT_THREADS) void radix_scatter(const uint32_t *__restrict__ keys_in,
                                                              const uint32_t *__restrict__ idx_in,
                                                              uint32_t *__restrict__ keys_out,
                                                              uint32_t *__restrict__ idx_out, int n, int shift,
                                                              const uint32_t *__restrict__ hist,
                                                              const uint32_t *__restrict__ dtot, int nblk)
{
    __shared__ uint32_t whist[4][256];   // per-wave running digit counts, later per-wave starts
    __shared__ uint32_t gbase[256];      // global start of (digit, this block)
    __shared__ uint32_t lstart[256];     // start of the digit inside the locally sorted tile
    __shared__ uint32_t dscan[4];
    __shared__ uint32_t skey[SORT_TILE], sidx[SORT_TILE];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
    for (int k = 0; k < 4; ++k) whist[k][tid] = 0;
    // exclusive scan of the 256 digit totals
    {
        int v = (int)dtot[tid], tot;
        int ex = wave_excl_scan(v, &tot);
        if (lane == 0) dscan[w] = (uint32_t)tot;
        __syncthreads();
        uint32_t wb = 0;
        for (int k = 0; k < w; ++k) wb += dscan[k];
        gbase[tid] = wb + (uint32_t)ex + hist[tid * nblk + blockIdx.x];
    }
    __syncthreads();
    const int tile0 = blockIdx.x * SORT_TILE;
    const int base = tile0 + w * (WAVE * SORT_ITEMS);
    uint32_t key[SORT_ITEMS], val[SORT_ITEMS], rank[SORT_ITEMS];
#pragma unroll
    for (int r = 0; r < SORT_ITEMS; ++r) {
        int e = base + r * WAVE + lane;
        bool valid = e < n;
        key[r] = valid ? keys_in[e] : 0u;
        val[r] = valid ? idx_in[e] : 0u;
        uint32_t d = (key[r] >> shift) & 0xFFu;
        // lanes of this round holding the same digit
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            uint64_t bal = __ballot((d >> b) & 1u);
            peers &= ((d >> b) & 1u) ? bal : ~bal;
        }
        uint32_t before = (uint32_t)__popcll(peers & lanemask_lt());
        uint32_t pre = whist[w][d];
        rank[r] = pre + before;
        __syncthreads();
        if (valid && before == 0) whist[w][d] = pre + (uint32_t)__popcll(peers);
        __syncthreads();
    }
    // per digit: where each wave's share starts inside the block's run, and where the run starts
    // inside the locally sorted tile
    {
        const uint32_t c0 = whist[0][tid], c1 = whist[1][tid], c2 = whist[2][tid], c3 = whist[3][tid];
        int tot;
        const int ex = wave_excl_scan((int)(c0 + c1 + c2 + c3), &tot);
        __syncthreads();
        if (lane == 0) dscan[w] = (uint32_t)tot;
        whist[0][tid] = 0; whist[1][tid] = c0; whist[2][tid] = c0 + c1; whist[3][tid] = c0 + c1 + c2;
        __syncthreads();
        uint32_t wb = 0;
        for (int k = 0; k < w; ++k) wb += dscan[k];
        lstart[tid] = wb + (uint32_t)ex;
    }
    __syncthreads();
    // stable local sort through LDS ...
#pragma unroll
    for (int r = 0; r < SORT_ITEMS; ++r) {
        int e = base + r * WAVE + lane;
        if (e < n) {
            uint32_t d = (key[r] >> shift) & 0xFFu;
            uint32_t lp = lstart[d] + whist[w][d] + rank[r];
            skey[lp] = key[r];
            sidx[lp] = val[r];
        }
    }
    __syncthreads();
    // ... so that consecutive threads write consecutive addresses within each digit's run
    const int cnt = min(SORT_TILE, n - tile0);
    for (int j = tid; j < cnt; j += SORT_THREADS) {
        const uint32_t k = skey[j];
        const uint32_t d = (k >> shift) & 0xFFu;
        const uint32_t pos = gbase[d] + ((uint32_t)j - lstart[d]);
        keys_out[pos] = k;
        idx_out[pos] = sidx[j];
    }
}

// ------------------------------------------------------------------ cells opened at each position
// The searches below are chains of dependent reads of the sorted keys, almost always within a
// few dozen positions of where they start.  Each workgroup therefore keeps the keys of its own
// positions plus a halo on both sides in LDS; reads outside that window go to memory.
constexpr int KEY_HALO = 256;

struct KeyWindow {
    const uint32_t *__restrict__ keys;   // sorted keys in memory
    const uint32_t *lds;                 // keys[lo, lo + len)
    uint32_t lo, len;
    __device__ __forceinline__ uint32_t operator[](uint32_t q) const
    {
        const uint32_t off = q - lo;
        return off < len ? lds[off] : keys[q];
    }
};

// Cooperative fill; the caller synchronises the workgroup afterwards.
__device__ __forceinline__ KeyWindow key_window_fill(const uint32_t *__restrict__ keys, uint32_t n, uint32_t first,
                                                     uint32_t count, uint32_t *lds)
{
    KeyWindow w;
    w.keys = keys;
    w.lds = lds;
    w.lo = first > (uint32_t)KEY_HALO ? first - KEY_HALO : 0u;
    const uint32_t hi = min(n, first + count + KEY_HALO);
    w.len = hi > w.lo ? hi - w.lo : 0u;
    for (uint32_t t = threadIdx.x; t < w.len; t += blockDim.x) lds[t] = keys[w.lo + t];
    return w;
}

// Sorted keys: the positions whose key shifted right by sh equals pre form one contiguous run.
__device__ __forceinline__ uint32_t run_end(const KeyWindow &keys, uint32_t n, uint32_t p, int sh, uint32_t pre)
{
    uint32_t lo = p, hi, step = 1;
    for (;;) {
        uint64_t cand = (uint64_t)p + step;
        if (cand >= n) { hi = n; break; }
        if ((keys[cand] >> sh) != pre) { hi = (uint32_t)cand; break; }
        lo = (uint32_t)cand;
        step <<= 1;
    }
    while (hi - lo > 1) {
        uint32_t mid = lo + ((hi - lo) >> 1);
        if ((keys[mid] >> sh) != pre) hi = mid; else lo = mid;
    }
    return hi;
}

__device__ __forceinline__ uint32_t run_begin(const KeyWindow &keys, uint32_t p, int sh, uint32_t pre)
{
    int64_t lo, hi = p, step = 1;
    for (;;) {
        int64_t cand = (int64_t)p - step;
        if (cand < 0) { lo = -1; break; }
        if ((keys[cand] >> sh) != pre) { lo = cand; break; }
        hi = cand;
        step <<= 1;
    }
    while (hi - lo > 1) {
        int64_t mid = lo + ((hi - lo) >> 1);
        if ((keys[mid] >> sh) != pre) lo = mid; else hi = mid;
    }
    return (uint32_t)hi;
}

// Depths [tmin, tend) of the cells that start at sorted position p.
__device__ __forceinline__ void levels_at(const KeyWindow &keys, uint32_t n, uint32_t p, int B,
                                          uint32_t C, int *tmin_out, int *tend_out)
{
    uint32_t key = keys[p];
    int tmin;
    if (p == 0) tmin = 0;
    else {
        uint32_t x = key ^ keys[p - 1];
        tmin = x ? B - ((31 - __clz((int)x)) >> 1) : B + 1;
    }
    int tend = tmin;
    if (tmin <= B) {
        uint32_t pc;   // number of points in the parent of the candidate cell
        if (tmin == 0) pc = 0xFFFFFFFFu;
        else if (tmin == 1) pc = n;
        else {
            int sh = 2 * (B - (tmin - 1));
            uint32_t pre = key >> sh;
            pc = run_end(keys, n, p, sh, pre) - run_begin(keys, p, sh, pre);
        }
        int t = tmin;
        while (t <= B && pc > C) {
            tend = t + 1;
            if (t == 0) pc = n;
            else {
                int sh = 2 * (B - t);
                pc = run_end(keys, n, p, sh, key >> sh) - p;
            }
            ++t;
        }
    }
    *tmin_out = tmin;
    *tend_out = tend;
}

// The same answer without any search when leaf_cap is small: the cell of depth s around p holds
// more than C points iff at least C of the 2C nearest positions (C on either side) share p's
// top s digits (L[j], R[j]: number of leading digits p shares with positions p-j, p+j).
constexpr int LEVELS_WINDOW_MAXC = 16;

__device__ __forceinline__ int common_digits(uint32_t a, uint32_t b, int B)
{
    const uint32_t x = a ^ b;
    return x ? B - 1 - ((31 - __clz((int)x)) >> 1) : B;
}

// CT > 0: leaf_cap known at compile time (all indices static, no bisection); CT = 0: any
// leaf_cap <= LEVELS_WINDOW_MAXC at run time.
template <int CT>
__device__ __forceinline__ void levels_window(const KeyWindow &keys, uint32_t n, uint32_t p, int B, int C,
                                              int *tmin_out, int *tend_out)
{
    const uint32_t key = keys[p];
    const int tmin = p == 0 ? 0 : (key == keys[p - 1] ? B + 1 : common_digits(key, keys[p - 1], B) + 1);
    int smax;
    if (CT > 0) {
        // C-th largest of the two non-increasing lists: max over k of min(L[k], R[CT - k]), with
        // L[0] = R[0] = B standing for "no neighbour needed on that side"
        int L[CT + 1], R[CT + 1];
        L[0] = R[0] = B;
#pragma unroll
        for (int j = 1; j <= CT; ++j) {
            L[j] = p >= (uint32_t)j ? common_digits(key, keys[p - j], B) : -1;
            R[j] = p + j < n ? common_digits(key, keys[p + j], B) : -1;
        }
        smax = -1;
#pragma unroll
        for (int k = 0; k <= CT; ++k) smax = max(smax, min(L[k], R[CT - k]));
    } else {
        int L[LEVELS_WINDOW_MAXC], R[LEVELS_WINDOW_MAXC];
#pragma unroll
        for (int j = 1; j <= LEVELS_WINDOW_MAXC; ++j) {
            L[j - 1] = (j <= C && p >= (uint32_t)j) ? common_digits(key, keys[p - j], B) : -1;
            R[j - 1] = (j <= C && p + j < n) ? common_digits(key, keys[p + j], B) : -1;
        }
        // deepest s in [0, B] with at least C of the 2C neighbours sharing s digits (-1 if none):
        // the count is non-increasing in s, so bisect
        int lo = -1, hi = B + 1;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            int cnt = 0;
#pragma unroll
            for (int j = 0; j < LEVELS_WINDOW_MAXC; ++j) cnt += (L[j] >= mid) + (R[j] >= mid);
            if (cnt >= C) lo = mid; else hi = mid;
        }
        smax = lo;
    }
    // cell (t, p) exists iff t == 0 or the depth t-1 cell around p holds more than C points
    int tend = min(B, smax + 1) + 1;
    if (tend < tmin) tend = tmin;
    *tmin_out = tmin;
    *tend_out = tend;
}

// Also moves the points into spatial order (step 4) and reduces each tile's (cells, sum x, sum y).
template <int CT>
__global__ __launch_bounds__(LEVEL_THREADS) void gather_levels(const float2 *__restrict__ Y,
                                                               const uint32_t *__restrict__ keys,
                                                               const uint32_t *__restrict__ perm, int n, int B, int C,
                                                               float2 *__restrict__ Ys, uint16_t *__restrict__ lev,
                                                               ScanPart *__restrict__ part)
{
    __shared__ double sx[4], sy[4];
    __shared__ uint32_t sc[4];
    __shared__ uint32_t kwin[LEVEL_TILE + 2 * KEY_HALO];
    const KeyWindow kw = key_window_fill(keys, (uint32_t)n, blockIdx.x * LEVEL_TILE, LEVEL_TILE, kwin);
    __syncthreads();
    double ax = 0.0, ay = 0.0;
    uint32_t ac = 0;
    float2 y[LEVEL_ITEMS];
#pragma unroll
    for (int k = 0; k < LEVEL_ITEMS; ++k) {
        const int p = blockIdx.x * LEVEL_TILE + k * LEVEL_THREADS + threadIdx.x;
        y[k] = p < n ? Y[min(perm[p], (uint32_t)n - 1u)] : make_float2(0.f, 0.f);
    }
#pragma unroll
    for (int k = 0; k < LEVEL_ITEMS; ++k) {
        const int p = blockIdx.x * LEVEL_TILE + k * LEVEL_THREADS + threadIdx.x;
        if (p < n) {
            Ys[p] = y[k];
            ax += (double)y[k].x; ay += (double)y[k].y;
            int tmin, tend;
            if (CT > 0 || C <= LEVELS_WINDOW_MAXC) levels_window<CT>(kw, (uint32_t)n, (uint32_t)p, B, C, &tmin, &tend);
            else levels_at(kw, (uint32_t)n, (uint32_t)p, B, (uint32_t)C, &tmin, &tend);
            lev[p] = (uint16_t)(tmin | (tend << 8));
            ac += (uint32_t)(tend - tmin);
        }
    }
    ax = wave_sum(ax); ay = wave_sum(ay); ac = wave_sum(ac);
    int w = threadIdx.x >> 6;
    if (lane_id() == 0) { sx[w] = ax; sy[w] = ay; sc[w] = ac; }
    __syncthreads();
    if (threadIdx.x == 0) {
        ScanPart q;
        q.sx = ((sx[0] + sx[1]) + sx[2]) + sx[3];
        q.sy = ((sy[0] + sy[1]) + sy[2]) + sy[3];
        q.cnt = sc[0] + sc[1] + sc[2] + sc[3];
        q.pad = 0;
        part[blockIdx.x] = q;
    }
}

// One block: exclusive prefix over the tile partials; total cell count to *ncells.
__global__ __launch_bounds__(1024) void scan_partials(ScanPart *__restrict__ part, int nparts,
                                                      uint32_t *__restrict__ ncells, uint32_t cap_cells,
                                                      uint32_t *status, uint32_t *__restrict__ big_count)
{
    if (threadIdx.x == 0) {
        big_count[0] = 0u;    // list of large cells filled by write_cells
    }
    if (threadIdx.x < WALK_COUNTERS) big_count[1 + threadIdx.x] = 0u;    // work counters of the walk
    __shared__ double wx[16], wy[16];
    __shared__ uint32_t wc[16];
    const int tid = threadIdx.x, w = tid >> 6;
    const int per = (nparts + 1023) / 1024;
    const int s = tid * per, e = min(nparts, s + per);
    double ax = 0.0, ay = 0.0;
    uint32_t ac = 0;
    for (int i = s; i < e; ++i) { ax += part[i].sx; ay += part[i].sy; ac += part[i].cnt; }
    // inclusive scan across the wave, then across the 16 waves
    double ix = ax, iy = ay;
    uint32_t icn = ac;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        double tx = __shfl_up(ix, o, WAVE), ty = __shfl_up(iy, o, WAVE);
        uint32_t tc = __shfl_up(icn, o, WAVE);
        if (lane_id() >= o) { ix += tx; iy += ty; icn += tc; }
    }
    if (lane_id() == WAVE - 1) { wx[w] = ix; wy[w] = iy; wc[w] = icn; }
    __syncthreads();
    double bx = 0.0, by = 0.0;
    uint32_t bc = 0;
    for (int k = 0; k < w; ++k) { bx += wx[k]; by += wy[k]; bc += wc[k]; }
    double px = bx + (ix - ax), py = by + (iy - ay);   // exclusive prefix of this thread's first item
    uint32_t pc = bc + (icn - ac);
    for (int i = s; i < e; ++i) {
        ScanPart q = part[i];
        ScanPart o;
        o.sx = px; o.sy = py; o.cnt = pc; o.pad = 0;
        part[i] = o;
        px += q.sx; py += q.sy; pc += q.cnt;
    }
    if (tid == 1023) {
        // thread 1023 holds the grand total whether or not it owned items
        *ncells = pc;
        if (pc > cap_cells) atomicOr(status, TSNE_STATUS_CELL_OVERFLOW);
    }
}

// Per position: index of the first cell opened there, and the running sums of the sorted
// coordinates (ps[p] = sum of Ys[0..p), ps[n] = total).
__global__ __launch_bounds__(LEVEL_THREADS) void downsweep(const float2 *__restrict__ Ys,
                                                           const uint16_t *__restrict__ lev, int n,
                                                           const ScanPart *__restrict__ part,
                                                           uint32_t *__restrict__ cellseq, double2 *__restrict__ ps,
                                                           uint32_t *__restrict__ cell_p, uint8_t *__restrict__ cell_t,
                                                           uint32_t cap_cells)
{
    __shared__ double wx[4], wy[4];
    __shared__ uint32_t wc[4];
    const int tid = threadIdx.x, w = tid >> 6;
    int p0 = blockIdx.x * LEVEL_TILE + tid * LEVEL_ITEMS;
    float2 y[LEVEL_ITEMS];
    uint32_t c[LEVEL_ITEMS], t0[LEVEL_ITEMS];
    double ax = 0.0, ay = 0.0;
    uint32_t ac = 0;
#pragma unroll
    for (int k = 0; k < LEVEL_ITEMS; ++k) {
        int p = p0 + k;
        if (p < n) {
            y[k] = Ys[p];
            uint32_t l = lev[p];
            c[k] = (l >> 8) - (l & 0xFFu);
            t0[k] = l & 0xFFu;
        } else { y[k] = make_float2(0.f, 0.f); c[k] = 0; t0[k] = 0; }
        ax += (double)y[k].x; ay += (double)y[k].y; ac += c[k];
    }
    double ix = ax, iy = ay;
    uint32_t icn = ac;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        double tx = __shfl_up(ix, o, WAVE), ty = __shfl_up(iy, o, WAVE);
        uint32_t tc = __shfl_up(icn, o, WAVE);
        if (lane_id() >= o) { ix += tx; iy += ty; icn += tc; }
    }
    if (lane_id() == WAVE - 1) { wx[w] = ix; wy[w] = iy; wc[w] = icn; }
    __syncthreads();
    ScanPart b = part[blockIdx.x];
    double px = b.sx, py = b.sy;
    uint32_t pc = b.cnt;
    for (int k = 0; k < w; ++k) { px += wx[k]; py += wy[k]; pc += wc[k]; }
    px += ix - ax; py += iy - ay; pc += icn - ac;
#pragma unroll
    for (int k = 0; k < LEVEL_ITEMS; ++k) {
        int p = p0 + k;
        if (p < n) {
            cellseq[p] = pc;
            ps[p] = make_double2(px, py);
            for (uint32_t q = 0; q < c[k]; ++q)
                if (pc + q < cap_cells) { cell_p[pc + q] = (uint32_t)p; cell_t[pc + q] = (uint8_t)(t0[k] + q); }
            px += (double)y[k].x; py += (double)y[k].y; pc += c[k];
            if (p == n - 1) { cellseq[n] = pc; ps[n] = make_double2(px, py); }
        }
    }
}

// First position in [s, e) whose digit (2 bits at sh) is >= q; e if none.
__device__ __forceinline__ uint32_t digit_lower_bound(const KeyWindow &keys, uint32_t s, uint32_t e,
                                                      int sh, uint32_t q)
{
    while (s < e) {
        uint32_t mid = s + ((e - s) >> 1);
        if (((keys[mid] >> sh) & 3u) < q) s = mid + 1; else e = mid;
    }
    return s;
}

// One lane per cell (cells are numbered in pre-order, so the cells of a workgroup start at
// non-decreasing positions and the keys they search sit in one short stretch, staged in LDS).
// A cell whose run of positions ends inside that stretch is finished on the spot.  The few large
// cells near the top of the tree would each be a chain of dozens of dependent memory reads in a
// single lane; they are put on a list instead and finished by write_big_cells, four lanes per cell.
constexpr int CELL_WINDOW = 4096;

__global__ __launch_bounds__(256) void write_cells(const uint32_t *__restrict__ keys,
                                                   const uint32_t *__restrict__ cellseq,
                                                   const double2 *__restrict__ ps,
                                                   const uint32_t *__restrict__ cell_p, const uint8_t *__restrict__ cell_t,
                                                   const uint32_t *__restrict__ ncells, int n, int B, int C,
                                                   Cell *__restrict__ cells, uint32_t cap_cells,
                                                   uint32_t *__restrict__ big_count, uint2 *__restrict__ big_list,
                                                   uint32_t big_cap)
{
    __shared__ uint32_t kwin[CELL_WINDOW];
    const uint32_t m = min(*ncells, cap_cells);
    for (uint32_t base = blockIdx.x * 256u; base < m; base += gridDim.x * 256u) {
        const uint32_t id = base + threadIdx.x;
        const bool live = id < m;
        const uint32_t p_first = cell_p[base], p_last = cell_p[min(base + 255u, m - 1u)];
        KeyWindow kw;
        kw.keys = keys;
        kw.lds = kwin;
        kw.lo = p_first;
        kw.len = min(min((uint32_t)n, p_last + 1u + (uint32_t)KEY_HALO) - p_first, (uint32_t)CELL_WINDOW);
        __syncthreads();                    // previous round's readers are done with the window
        for (uint32_t q = threadIdx.x; q < kw.len; q += 256u) kwin[q] = keys[p_first + q];
        __syncthreads();
        if (!live) continue;
        const uint32_t p = cell_p[id];
        const int t = (int)cell_t[id];
        const uint32_t key = kw[p];
        const uint32_t wend = kw.lo + kw.len;                  // one past the last position in the window
        if (p < wend && wend < (uint32_t)n &&
            (t == 0 || (kwin[kw.len - 1] >> (2 * (B - t))) == (key >> (2 * (B - t))))) {
            // the cell runs past the window: a large cell
            const uint32_t slot = atomicAdd(big_count, 1u);
            if (slot < big_cap) { big_list[slot] = make_uint2(p, (uint32_t)t); continue; }
            // list full (cannot happen for capacity n/8 + 1024 unless most cells are huge): finish it here
        }
        const uint32_t e = (t == 0) ? (uint32_t)n : run_end(kw, (uint32_t)n, p, 2 * (B - t), key >> (2 * (B - t)));
        const uint32_t cnt = e - p;
        const double2 s0 = ps[p], s1 = ps[e];
        Cell c;
        c.cx = (float)((s1.x - s0.x) / (double)cnt);
        c.cy = (float)((s1.y - s0.y) / (double)cnt);
        c.cnt = cnt;
        const bool leaf = cnt <= (uint32_t)C || t == B;
        c.meta = (uint32_t)t | (leaf ? 0x100u : 0u);
        c.lo = p;
        c.c1 = c.c2 = c.c3 = TSNE_NONE;
        if (!leaf) {
            const int sh = 2 * (B - t - 1);
            uint32_t kids[3];
            int nk = 0;
            uint32_t s = p;
            const uint32_t qfirst = (key >> sh) & 3u;
            for (uint32_t q = qfirst + 1; q < 4; ++q) {
                const uint32_t b = digit_lower_bound(kw, s, e, sh, q);
                if (b < e && ((kw[b] >> sh) & 3u) == q) kids[nk++] = cellseq[b];
                s = b;
            }
            if (nk > 0) c.c1 = kids[0];
            if (nk > 1) c.c2 = kids[1];
            if (nk > 2) c.c3 = kids[2];
        }
        cells[id] = c;
    }
}

// First position x in [lo, n) with (keys[x] >> sh) >= target, n if none (keys sorted).
// First position i in [lo, n) with (keys[i] >> sh) >= target (n if there is none), found by the
// whole wave: every round the 64 lanes probe 64 evenly spaced positions of the remaining range,
// which shrinks 64-fold, so four rounds cover any n.  All lanes must call with the same
// arguments; every probed index lies inside [lo, n) whatever the keys hold.
__device__ __forceinline__ uint32_t wave_shifted_lower_bound(const uint32_t *__restrict__ keys, uint32_t lo, uint32_t n,
                                                             int sh, uint64_t target)
{
    uint32_t hi = n;
    const uint32_t lane = (uint32_t)lane_id();
    while (lo < hi) {
        const uint32_t step = (hi - lo + 63u) >> 6;
        const uint64_t probe = (uint64_t)lo + (uint64_t)(lane + 1u) * step - 1ull;
        bool below = false;
        if (probe < (uint64_t)hi) below = (uint64_t)(keys[probe] >> sh) < target;
        const uint32_t c = (uint32_t)__popcll(__ballot(below));   // the keys are sorted: lanes 0..c-1
        const uint64_t top = (uint64_t)lo + (uint64_t)(c + 1u) * step - 1ull;
        lo += c * step;
        hi = top < (uint64_t)hi ? (uint32_t)top : hi;
    }
    return lo;
}

// One workgroup per listed cell, one wave per search: wave 0 finds the end of the cell, waves
// 1-3 the first position of quadrants 1-3 among its points (all four are lower bounds in the
// globally sorted keys).
__global__ __launch_bounds__(256) void write_big_cells(const uint32_t *__restrict__ keys, const uint16_t *__restrict__ lev,
                                                       const uint32_t *__restrict__ cellseq,
                                                       const double2 *__restrict__ ps, int n, int B, int C,
                                                       Cell *__restrict__ cells, uint32_t cap_cells,
                                                       const uint32_t *__restrict__ big_count,
                                                       const uint2 *__restrict__ big_list, uint32_t big_cap)
{
    __shared__ uint32_t found_s[4];
    const int role = (int)(threadIdx.x >> 6);
    const uint32_t m = min(*big_count, big_cap);
    for (uint32_t item = blockIdx.x; item < m; item += gridDim.x) {
        const uint2 it = big_list[item];
        const uint32_t p = min(it.x, (uint32_t)n - 1u);
        const int t = min((int)it.y, B);
        const uint32_t key = keys[p];
        uint32_t found = (uint32_t)n;
        if (role == 0) {
            if (t > 0) {
                const int sh = 2 * (B - t);
                found = wave_shifted_lower_bound(keys, p, (uint32_t)n, sh, (uint64_t)(key >> sh) + 1ull);
            }
        } else if (t < B) {
            const int sh = 2 * (B - t - 1);
            const uint64_t parent = t > 0 ? (uint64_t)(key >> (2 * (B - t))) : 0ull;
            found = wave_shifted_lower_bound(keys, p, (uint32_t)n, sh, (parent << 2) + (uint64_t)role);
        }
        if (lane_id() == 0) found_s[role] = found;
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t e = found_s[0];
            const uint32_t b1 = min(found_s[1], e), b2 = min(found_s[2], e), b3 = min(found_s[3], e);
            const uint32_t l = lev[p];
            const uint32_t id = cellseq[p] + (uint32_t)(t - (int)(l & 0xFFu));
            if (id < cap_cells) {
                const uint32_t cnt = e - p;
                const double2 s0 = ps[p], s1 = ps[e];
                Cell c;
                c.cx = (float)((s1.x - s0.x) / (double)cnt);
                c.cy = (float)((s1.y - s0.y) / (double)cnt);
                c.cnt = cnt;
                const bool leaf = cnt <= (uint32_t)C || t == B;
                c.meta = (uint32_t)t | (leaf ? 0x100u : 0u);
                c.lo = p;
                c.c1 = c.c2 = c.c3 = TSNE_NONE;
                if (!leaf) {
                    // quadrant q > first quadrant exists iff its first position precedes the next boundary
                    const uint32_t qfirst = (key >> (2 * (B - t - 1))) & 3u;
                    const uint32_t bnd[5] = {p, b1, b2, b3, e};
                    uint32_t kids[3];
                    int nk = 0;
                    for (uint32_t q = qfirst + 1; q < 4; ++q)
                        if (bnd[q] < bnd[q + 1]) kids[nk++] = cellseq[bnd[q]];
                    if (nk > 0) c.c1 = kids[0];
                    if (nk > 1) c.c2 = kids[1];
                    if (nk > 2) c.c3 = kids[2];
                }
                cells[id] = c;
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ export (tests only)
__global__ void export_cells_k(const Cell *__restrict__ cells, const uint32_t *__restrict__ ncells, int cap,
                               int32_t *depth, int32_t *lo, int32_t *hi, int32_t *leaf, float *com)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    int m = (int)min(*ncells, (uint32_t)cap);
    if (i >= m) return;
    Cell c = cells[i];
    if (depth) depth[i] = (int32_t)(c.meta & 0xFFu);
    if (lo) lo[i] = (int32_t)c.lo;
    if (hi) hi[i] = (int32_t)(c.lo + c.cnt);
    if (leaf) leaf[i] = (int32_t)((c.meta >> 8) & 1u);
    if (com) { com[2 * i] = c.cx; com[2 * i + 1] = c.cy; }
}

hipError_t launch_export_cells(tsne_ctx *c, int32_t cap, int32_t *depth, int32_t *lo, int32_t *hi, int32_t *leaf,
                               float *com, hipStream_t s)
{
    if (cap <= 0) return hipSuccess;
    int m = cap < c->cap_cells ? cap : c->cap_cells;
    hipLaunchKernelGGL(export_cells_k, dim3((m + 255) / 256), dim3(256), 0, s, c->cells, c->ncells, m, depth, lo, hi,
                       leaf, com);
    return hipGetLastError();
}

// ------------------------------------------------------------------ host: enqueue the whole build
static int bbox_blocks(int n)
{
    int nb = (n + 255) / 256;
    return nb < BBOX_MAX_BLOCKS ? nb : BBOX_MAX_BLOCKS;
}

// Stable LSD radix sort of (keys[0], idx[0]) on the low nbits bits, 8 bits a pass.
hipError_t launch_sort(tsne_ctx *c, int nbits, hipStream_t s)
{
    const int n = c->p.n;
    const int nblk = (n + SORT_TILE - 1) / SORT_TILE;
    int cur = 0;
    for (int shift = 0; shift < nbits; shift += 8) {
        hipLaunchKernelGGL(radix_hist, dim3(nblk), dim3(SORT_THREADS), 0, s, c->keys[cur], n, shift, c->hist, nblk);
        hipLaunchKernelGGL(radix_scan, dim3(256), dim3(256), 0, s, c->hist, nblk, c->dtot);
        hipLaunchKernelGGL(radix_scatter, dim3(nblk), dim3(SORT_THREADS), 0, s, c->keys[cur], c->idx[cur],
                           c->keys[cur ^ 1], c->idx[cur ^ 1], n, shift, c->hist, c->dtot, nblk);
        cur ^= 1;
    }
    c->sorted_buf = cur;
    return hipGetLastError();
}

// Step 1, first half: the caller's Y into slot order plus per-block bounding boxes.
hipError_t launch_gather_bbox(tsne_ctx *c, const float *d_Y, hipStream_t s)
{
    const int n = c->p.n;
    hipLaunchKernelGGL(bbox_partial, dim3(bbox_blocks(n)), dim3(256), 0, s, (const float2 *)d_Y,
                       c->orig[c->cur_state], c->Yi, n, c->bbox_part, c->status);
    c->bbox_nparts = bbox_blocks(n);
    return hipGetLastError();
}

// Step 1 second half, step 2a and step 4: root square, keys, spatial sort.
hipError_t launch_tree_sort(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n, B = c->p.morton_bits;
    const float2 *Y = c->Yi;
    const int nb = (n + 255) / 256;
    if (n <= SMALL_SORT_MAX) {
        int m = 512;
        while (m < n) m <<= 1;
        const int cur = ((2 * B + 7) / 8) & 1;     // where the radix passes would have left the result
        hipLaunchKernelGGL(small_root_keys_sort<3>, dim3(1), dim3(m >> 3), small_sort_lds(m), s, Y, n, m, c->bbox_part,
                           c->bbox_nparts, B, c->root, c->keys_orig, c->keys[cur], c->idx[cur], c->status);
        c->sorted_buf = cur;
        return hipGetLastError();
    }
    hipLaunchKernelGGL(bbox_final, dim3(1), dim3(c->bbox_nparts > 1024 ? 1024 : 256), 0, s, c->bbox_part, c->bbox_nparts, B,
                       c->root, c->status);
    hipLaunchKernelGGL(morton_encode, dim3(nb), dim3(256), 0, s, Y, n, c->root, B, c->keys_orig, c->keys[0],
                       c->idx[0]);
    return launch_sort(c, 2 * B, s);
}

// Steps 2b, 2c and 3: cells, counts, centres of mass from the sorted keys.
hipError_t launch_tree_cells(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n, B = c->p.morton_bits, C = c->p.leaf_cap;
    const float2 *Y = c->Yi;
    const int nb = (n + 255) / 256;
    const int cur = c->sorted_buf;
    int nl = (n + LEVEL_TILE - 1) / LEVEL_TILE;
    if (C == 8)
        hipLaunchKernelGGL(gather_levels<8>, dim3(nl), dim3(LEVEL_THREADS), 0, s, Y, c->keys[cur], c->idx[cur], n, B,
                           C, c->Ys, c->lev, c->part);
    else
        hipLaunchKernelGGL(gather_levels<0>, dim3(nl), dim3(LEVEL_THREADS), 0, s, Y, c->keys[cur], c->idx[cur], n, B,
                           C, c->Ys, c->lev, c->part);
    hipLaunchKernelGGL(scan_partials, dim3(1), dim3(1024), 0, s, c->part, nl, c->ncells, (uint32_t)c->cap_cells,
                       c->status, c->big_count);
    hipLaunchKernelGGL(downsweep, dim3(nl), dim3(LEVEL_THREADS), 0, s, c->Ys, c->lev, n, c->part, c->cellseq, c->ps,
                       c->cell_p, c->cell_t, (uint32_t)c->cap_cells);
    // grid sized for n cells (a typical tree has about n / 3); the kernel strides if there are more
    hipLaunchKernelGGL(write_cells, dim3(nb), dim3(256), 0, s, c->keys[cur], c->cellseq, c->ps, c->cell_p, c->cell_t,
                       c->ncells, n, B, C, c->cells, (uint32_t)c->cap_cells, c->big_count, c->big_list,
                       (uint32_t)c->big_cap);
    hipLaunchKernelGGL(write_big_cells, dim3(4096), dim3(256), 0, s, c->keys[cur], c->lev,
                       c->cellseq, c->ps, n, B, C, c->cells, (uint32_t)c->cap_cells, c->big_count, c->big_list,
                       (uint32_t)c->big_cap);
    return hipGetLastError();
}
