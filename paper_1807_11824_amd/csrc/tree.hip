// Sec. III-C steps 1-4 of the paper on gfx950: bounding box, grid keys, spatial sort,
// quad tree and cell summaries.  Nothing here walks pointers or inserts points one by one:
// the tree is read off the sorted keys.
//
//   bbox_partial / bbox_final   step 1   min/max reduction -> root square (power-of-two side)
//   morton_encode_hist          step 2a  grid coordinates (up to 24 bits per axis), bit-interleaved key
//   radix_hist / _scan / _scatter  step 4  stable LSD radix sort, 11 bits a pass
//   small_root_keys_sort        steps 1, 2a, 4 in one launch of one workgroup, for few points
//   gather_levels               step 2b  which cells start at each sorted position
//   downsweep                   step 3   prefix sums: cell numbering and running coordinate sums
//   write_cells                 steps 2c+3  cell records: members, count, centre of mass, children
//
// The sort works on one 64-bit word per point, (key << key_shift) | slot with key_shift = 64 - 2 bits:
// the order of the words is the order by (key, slot), which is the stable order the tree is defined
// on, and no index array travels through the passes.
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
// bits of v (up to 24) to the even positions
__device__ __forceinline__ uint64_t spread24(uint32_t q)
{
    uint64_t v = q & 0xFFFFFFu;
    v = (v | (v << 16)) & 0x0000FFFF0000FFFFull;
    v = (v | (v << 8)) & 0x00FF00FF00FF00FFull;
    v = (v | (v << 4)) & 0x0F0F0F0F0F0F0F0Full;
    v = (v | (v << 2)) & 0x3333333333333333ull;
    v = (v | (v << 1)) & 0x5555555555555555ull;
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

__device__ __forceinline__ uint64_t grid_key(float2 y, float4 r, uint32_t qmax)
{
    return spread24(grid_coord(y.x, r.x, r.w, qmax)) | (spread24(grid_coord(y.y, r.y, r.w, qmax)) << 1);
}

// ------------------------------------------------------------------ few points: one workgroup does it all
// Root square, keys and the sort in one launch, for n <= SMALL_SORT_MAX: the words (key, slot) sit
// in LDS (all different, so any sorting network gives the order of a stable sort by key), padded
// with all-ones to m, the power of two >= n.  Same root, same keys and same order as bbox_final +
// morton_encode_hist + the radix passes.
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
                                                             int ks, float4 *__restrict__ root,
                                                             uint64_t *__restrict__ words_out, uint32_t *status)
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
        if (i < n) v = (grid_key(Y[i], r, qmax) << ks) | (uint32_t)i;
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
    for (int i = tid; i < n; i += nthr) words_out[i] = pairs[small_sort_slot(i)];
}

static size_t small_sort_lds(int m) { return 8 * (size_t)(m + (m >> 3)); }

hipError_t small_sort_prepare()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&small_root_keys_sort<3>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)small_sort_lds(SMALL_SORT_MAX));
}

// ------------------------------------------------------------------ radix sort (stable, LSD, 11 bits a pass)
// Three kernels a pass: digit counts per tile (hist[tile][digit]; the first pass gets them from
// the kernel that wrote the words), their prefix over the tiles, and the scatter.
__device__ __forceinline__ uint32_t digit_of(uint64_t w, int lo, uint32_t mask) { return (uint32_t)(w >> lo) & mask; }

// Root square (already reduced), grid key and word of every point, and the digit counts of the
// first radix pass.
// (ITEMS words per thread: the tile size is chosen per context, see sort_items())
template <int ITEMS>
__global__ __launch_bounds__(SORT_THREADS) void morton_encode_hist(const float2 *__restrict__ Y, int n,
                                                                   const float4 *__restrict__ root, int bits, int ks,
                                                                   uint32_t mask, uint64_t *__restrict__ words,
                                                                   uint32_t *__restrict__ hist, int nblk)
{
    __shared__ uint32_t h[RADIX];
    for (int d = threadIdx.x; d < RADIX; d += SORT_THREADS) h[d] = 0u;
    __syncthreads();
    const float4 r = *root;
    const uint32_t qmax = (1u << bits) - 1u;
    const int base = blockIdx.x * (SORT_THREADS * ITEMS);
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int e = base + k * SORT_THREADS + (int)threadIdx.x;
        if (e < n) {
            const uint64_t w = (grid_key(Y[e], r, qmax) << ks) | (uint32_t)e;
            words[e] = w;
            atomicAdd(&h[digit_of(w, ks, mask)], 1u);
        }
    }
    __syncthreads();
    for (int d = threadIdx.x; d < RADIX; d += SORT_THREADS) hist[(size_t)blockIdx.x * RADIX + d] = h[d];
}

template <int ITEMS>
__global__ __launch_bounds__(SORT_THREADS) void radix_hist(const uint64_t *__restrict__ words, int n, int lo, uint32_t mask,
                                                           uint32_t *__restrict__ hist, int nblk)
{
    __shared__ uint32_t h[RADIX];
    for (int d = threadIdx.x; d < RADIX; d += SORT_THREADS) h[d] = 0u;
    __syncthreads();
    const int base = blockIdx.x * (SORT_THREADS * ITEMS);
    uint64_t w[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {          // all loads in flight before the first count
        const int e = base + k * SORT_THREADS + (int)threadIdx.x;
        w[k] = e < n ? words[e] : 0ull;
    }
#pragma unroll
    for (int k = 0; k < ITEMS; ++k)
        if (base + k * SORT_THREADS + (int)threadIdx.x < n) atomicAdd(&h[digit_of(w[k], lo, mask)], 1u);
    __syncthreads();
    for (int d = threadIdx.x; d < RADIX; d += SORT_THREADS) hist[(size_t)blockIdx.x * RADIX + d] = h[d];
}

// hist[t][d] becomes the number of words with digit d in tiles before t; dtot[d] the digit's total.
// A workgroup takes SCAN_DIGITS neighbouring digits; SCAN_SEGS threads share a digit, each a segment of
// the tiles, whose counts it loads in batches (so that its loads are in flight together).
constexpr int SCAN_DIGITS = 16, SCAN_SEGS = 64, SCAN_BATCH = 8;
__global__ __launch_bounds__(SCAN_DIGITS * SCAN_SEGS) void radix_scan(uint32_t *__restrict__ hist, int nblk,
                                                                      uint32_t *__restrict__ dtot)
{
    __shared__ uint32_t ssum[SCAN_SEGS][SCAN_DIGITS];
    const int dl = (int)threadIdx.x % SCAN_DIGITS, sg = (int)threadIdx.x / SCAN_DIGITS;
    const int d = blockIdx.x * SCAN_DIGITS + dl;
    const int len = (nblk + SCAN_SEGS - 1) / SCAN_SEGS;
    const int t0 = min(nblk, sg * len), t1 = min(nblk, t0 + len);
    uint32_t sum = 0;
    for (int tb = t0; tb < t1; tb += SCAN_BATCH) {
        uint32_t v[SCAN_BATCH];
#pragma unroll
        for (int k = 0; k < SCAN_BATCH; ++k) v[k] = tb + k < t1 ? hist[(size_t)(tb + k) * RADIX + d] : 0u;
#pragma unroll
        for (int k = 0; k < SCAN_BATCH; ++k) sum += v[k];
    }
    ssum[sg][dl] = sum;
    __syncthreads();
    uint32_t run = 0, all = 0;
    for (int k = 0; k < SCAN_SEGS; ++k) {
        const uint32_t v = ssum[k][dl];
        run += k < sg ? v : 0u;
        all += v;
    }
    if (sg == 0) dtot[d] = all;
    for (int tb = t0; tb < t1; tb += SCAN_BATCH) {
        uint32_t v[SCAN_BATCH];
#pragma unroll
        for (int k = 0; k < SCAN_BATCH; ++k) v[k] = tb + k < t1 ? hist[(size_t)(tb + k) * RADIX + d] : 0u;
#pragma unroll
        for (int k = 0; k < SCAN_BATCH; ++k) {
            if (tb + k < t1) hist[(size_t)(tb + k) * RADIX + d] = run;
            run += v[k];
        }
    }
}

// Exclusive prefix over the workgroup of one value per thread (SORT_THREADS threads); all threads call.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *wsum /* SORT_THREADS / 64 */)
{
    int tot;
    const int ex = wave_excl_scan((int)v, &tot);
    const int w = (int)threadIdx.x >> 6;
    __syncthreads();
    if (lane_id() == 0) wsum[w] = (uint32_t)tot;
    __syncthreads();
    uint32_t wb = 0;
    for (int k = 0; k < w; ++k) wb += wsum[k];
    return wb + (uint32_t)ex;
}

// Workgroups reach the eight XCDs in turn.  Tile numbers are dealt so that each XCD works on a
// contiguous range of tiles: the pieces of one digit's output run that neighbouring tiles write
// are adjacent in memory, and this way they meet in one second-level cache and leave it as whole lines.
__device__ __forceinline__ int scatter_tile(int block, int nblk)
{
    const int per = (nblk + 7) / 8;
    return (block % 8) * per + block / 8;
}

template <int ITEMS>
__global__ __launch_bounds__(SORT_THREADS) void radix_scatter(const uint64_t *__restrict__ in, uint64_t *__restrict__ out,
                                                              int n, int lo, uint32_t mask,
                                                              const uint32_t *__restrict__ hist,
                                                              const uint32_t *__restrict__ dtot, int nblk)
{
    constexpr int NW = SORT_THREADS / WAVE, DPT = RADIX / SORT_THREADS;   // digits per thread
    constexpr int TILE = SORT_THREADS * ITEMS;
    // per-wave running digit counts, later per-wave starts; once every word knows its place in the
    // locally sorted tile the same memory holds that tile
    constexpr size_t OVERLAY = sizeof(uint16_t) * NW * RADIX > (size_t)TILE * 8 ? sizeof(uint16_t) * NW * RADIX
                                                                                   : (size_t)TILE * 8;
    __shared__ __align__(16) unsigned char overlay[OVERLAY];
    uint16_t (*whist)[RADIX] = reinterpret_cast<uint16_t (*)[RADIX]>(overlay);
    uint64_t *sorted = reinterpret_cast<uint64_t *>(overlay);
    __shared__ uint32_t gbase[RADIX];       // global start of (digit, this tile)
    __shared__ uint16_t lstart[RADIX];      // start of the digit inside the locally sorted tile
    __shared__ uint32_t wsum[NW];
    const int tile = scatter_tile((int)blockIdx.x, nblk);
    if (tile >= nblk) return;               // the same for every thread of the workgroup
    const int tid = (int)threadIdx.x, w = tid >> 6, lane = tid & 63;
    const int tile0 = tile * TILE;
    const int base = tile0 + w * (WAVE * ITEMS);
    uint64_t word[ITEMS];
    uint32_t rank[ITEMS];
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {       // requested first: they arrive while the offsets below are worked out
        const int e = base + r * WAVE + lane;
        word[r] = e < n ? in[e] : 0ull;
    }
    {
        uint32_t *z = reinterpret_cast<uint32_t *>(overlay);
        for (int i = tid; i < NW * RADIX / 2; i += SORT_THREADS) z[i] = 0u;
    }
    // where every digit's run starts in the output: digits before it, then tiles before this one
    {
        uint32_t t[DPT], before[DPT], sum = 0;
#pragma unroll
        for (int j = 0; j < DPT; ++j) {
            t[j] = dtot[tid * DPT + j];
            before[j] = hist[(size_t)tile * RADIX + tid * DPT + j];
            sum += t[j];
        }
        uint32_t run = block_excl_scan(sum, wsum);      // (its barriers also cover the zeroing above)
#pragma unroll
        for (int j = 0; j < DPT; ++j) {
            gbase[tid * DPT + j] = run + before[j];
            run += t[j];
        }
    }
    // Rank inside the wave's share, one item of every lane at a time: lanes with the same digit are
    // found with one ballot per digit bit.  whist[w] is touched by wave w alone, whose LDS
    // instructions execute in program order, so the rounds need no barrier between them.
    volatile uint16_t *mine = whist[w];
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const bool valid = base + r * WAVE + lane < n;
        const uint32_t d = digit_of(word[r], lo, mask);
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < RADIX_BITS; ++b) {
            const uint64_t bal = __ballot((d >> b) & 1u);
            peers &= ((d >> b) & 1u) ? bal : ~bal;
        }
        const uint32_t before = (uint32_t)__popcll(peers & lanemask_lt());
        const uint32_t pre = mine[d];
        rank[r] = pre + before;
        if (valid && before == 0) mine[d] = (uint16_t)(pre + (uint32_t)__popcll(peers));
    }
    __syncthreads();
    // per digit: where each wave's share starts inside the tile's run, and where the run starts
    // inside the locally sorted tile
    {
        uint32_t tot[DPT], sum = 0;
#pragma unroll
        for (int j = 0; j < DPT; ++j) {
            uint32_t acc = 0;
#pragma unroll
            for (int k = 0; k < NW; ++k) {
                const uint32_t c = whist[k][tid * DPT + j];
                whist[k][tid * DPT + j] = (uint16_t)acc;
                acc += c;
            }
            tot[j] = acc;
            sum += acc;
        }
        uint32_t run = block_excl_scan(sum, wsum);
#pragma unroll
        for (int j = 0; j < DPT; ++j) { lstart[tid * DPT + j] = (uint16_t)run; run += tot[j]; }
    }
    __syncthreads();
    // stable local sort through LDS ...
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const uint32_t d = digit_of(word[r], lo, mask);
        rank[r] += (uint32_t)lstart[d] + (uint32_t)whist[w][d];
    }
    __syncthreads();      // the counts are no longer needed: their memory becomes the sorted tile
#pragma unroll
    for (int r = 0; r < ITEMS; ++r)
        if (base + r * WAVE + lane < n) sorted[min(rank[r], (uint32_t)TILE - 1u)] = word[r];
    __syncthreads();
    // ... so that consecutive threads write consecutive addresses within each digit's run
    const int cnt = min(TILE, n - tile0);
    for (int j = tid; j < cnt; j += SORT_THREADS) {
        const uint64_t v = sorted[j];
        const uint32_t d = digit_of(v, lo, mask);
        const uint32_t pos = gbase[d] + ((uint32_t)j - (uint32_t)lstart[d]);
        if (pos < (uint32_t)n) out[pos] = v;
    }
}

// the low 32 bits of every word
__global__ __launch_bounds__(256) void unpack_perm_k(const uint64_t *__restrict__ words, int n, uint32_t *__restrict__ perm)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) perm[p] = (uint32_t)words[p];
}

// ------------------------------------------------------------------ cells opened at each position
// The searches below are chains of dependent reads of the sorted keys, almost always within a
// few dozen positions of where they start.  Each workgroup therefore keeps the keys of its own
// positions plus a halo on both sides in LDS; reads outside that window go to memory.
constexpr int KEY_HALO = 256;

struct KeyWindow {
    const uint64_t *__restrict__ words;  // sorted words in memory (key << ks | slot)
    const uint64_t *lds;                 // keys of positions [lo, lo + len)
    uint32_t lo, len;
    int ks;
    __device__ __forceinline__ uint64_t operator[](uint32_t q) const
    {
        const uint32_t off = q - lo;
        return off < len ? lds[off] : words[q] >> ks;
    }
};

// Keys of positions [lo, ...) in LDS, for searches that are known to stay inside.
struct LdsKeys {
    const uint64_t *lds;
    uint32_t lo;
    __device__ __forceinline__ uint64_t operator[](uint32_t q) const { return lds[q - lo]; }
};

// Cooperative fill; the caller synchronises the workgroup afterwards.
__device__ __forceinline__ KeyWindow key_window_fill(const uint64_t *__restrict__ words, int ks, uint32_t n, uint32_t first,
                                                     uint32_t count, uint64_t *lds)
{
    KeyWindow w;
    w.words = words;
    w.lds = lds;
    w.ks = ks;
    w.lo = first > (uint32_t)KEY_HALO ? first - KEY_HALO : 0u;
    const uint32_t hi = min(n, first + count + KEY_HALO);
    w.len = hi > w.lo ? hi - w.lo : 0u;
    for (uint32_t t = threadIdx.x; t < w.len; t += blockDim.x) lds[t] = words[w.lo + t] >> ks;
    return w;
}

// Sorted keys: the positions whose key shifted right by sh equals pre form one contiguous run.
template <class Keys>
__device__ __forceinline__ uint32_t run_end(const Keys &keys, uint32_t n, uint32_t p, int sh, uint64_t pre)
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

__device__ __forceinline__ uint32_t run_begin(const KeyWindow &keys, uint32_t p, int sh, uint64_t pre)
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
    uint64_t key = keys[p];
    int tmin;
    if (p == 0) tmin = 0;
    else {
        uint64_t x = key ^ keys[p - 1];
        tmin = x ? B - ((63 - __clzll((long long)x)) >> 1) : B + 1;
    }
    int tend = tmin;
    if (tmin <= B) {
        uint32_t pc;   // number of points in the parent of the candidate cell
        if (tmin == 0) pc = 0xFFFFFFFFu;
        else if (tmin == 1) pc = n;
        else {
            int sh = 2 * (B - (tmin - 1));
            uint64_t pre = key >> sh;
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

__device__ __forceinline__ int common_digits(uint64_t a, uint64_t b, int B)
{
    const uint64_t x = a ^ b;
    return x ? B - 1 - ((63 - __clzll((long long)x)) >> 1) : B;
}

// The keys are sorted, so the digits p shares with p+j are the fewest shared by any two
// neighbours in between: with adj[q] = digits shared by positions q and q+1 (-1 beyond either end
// of the array), R[j] = min(adj[p], .., adj[p+j-1]) and L[j] = min(adj[p-1], .., adj[p-j]).  Every
// workgroup works adj out once for its positions and a margin (one 64-bit comparison per position),
// after which a position needs 2C byte reads and minima.
// CT > 0: leaf_cap known at compile time (all indices static, no bisection); CT = 0: any
// leaf_cap <= LEVELS_WINDOW_MAXC at run time.  adj points at the entry of position p.
template <int CT>
__device__ __forceinline__ void levels_window(const signed char *adj, int B, int C, int *tmin_out, int *tend_out)
{
    const int prev = adj[-1];
    const int tmin = prev == B ? B + 1 : prev + 1;       // (position 0: adj[-1] = -1, depth 0)
    int smax;
    if (CT > 0) {
        // C-th largest of the two non-increasing lists: max over k of min(L[k], R[CT - k]), with
        // L[0] = R[0] = B standing for "no neighbour needed on that side"
        int L[CT + 1], R[CT + 1];
        L[0] = R[0] = B;
#pragma unroll
        for (int j = 1; j <= CT; ++j) {
            L[j] = min(L[j - 1], (int)adj[-j]);
            R[j] = min(R[j - 1], (int)adj[j - 1]);
        }
        smax = -1;
#pragma unroll
        for (int k = 0; k <= CT; ++k) smax = max(smax, min(L[k], R[CT - k]));
    } else {
        int L[LEVELS_WINDOW_MAXC], R[LEVELS_WINDOW_MAXC];
        int l = B, r = B;
#pragma unroll
        for (int j = 1; j <= LEVELS_WINDOW_MAXC; ++j) {
            l = min(l, (int)adj[-j]);
            r = min(r, (int)adj[j - 1]);
            L[j - 1] = j <= C ? l : -1;
            R[j - 1] = j <= C ? r : -1;
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

// Also moves the points into spatial order (step 4), writes the order itself (position -> slot)
// and reduces each tile's (cells, sum x, sum y).  CT < 0: any leaf_cap, by searching the keys.
template <int CT>
__global__ __launch_bounds__(LEVEL_THREADS) void gather_levels(const float2 *__restrict__ Y,
                                                               const uint64_t *__restrict__ words, int ks, int n, int B,
                                                               int C, float2 *__restrict__ Ys,
                                                               uint32_t *__restrict__ perm, uint16_t *__restrict__ lev,
                                                               ScanPart *__restrict__ part,
                                                               uint32_t *__restrict__ counters)
{
    __shared__ double sx[4], sy[4];
    __shared__ uint32_t sc[4];
    constexpr int MARGIN = LEVELS_WINDOW_MAXC + 1;
    __shared__ uint64_t kwin[CT < 0 ? LEVEL_TILE + 2 * KEY_HALO : 1];
    __shared__ signed char adjw[CT < 0 ? 1 : LEVEL_TILE + 2 * MARGIN];
    // the list of large cells (write_cells) and the work counters of the walk start at zero
    if (blockIdx.x == 0 && threadIdx.x < 1 + WALK_COUNTERS) counters[threadIdx.x] = 0u;
    const int first = blockIdx.x * LEVEL_TILE;
    KeyWindow kw;
    if (CT < 0) {
        kw = key_window_fill(words, ks, (uint32_t)n, (uint32_t)first, LEVEL_TILE, kwin);
    } else {
        // adjw[i]: digits shared by positions q = first - MARGIN + i and q + 1
        for (int i = threadIdx.x; i < LEVEL_TILE + 2 * MARGIN; i += LEVEL_THREADS) {
            const int q = first - MARGIN + i;
            adjw[i] = (q < 0 || q + 1 >= n) ? (signed char)-1
                                            : (signed char)common_digits(words[q] >> ks, words[q + 1] >> ks, B);
        }
    }
    double ax = 0.0, ay = 0.0;
    uint32_t ac = 0;
    float2 y[LEVEL_ITEMS];
#pragma unroll
    for (int k = 0; k < LEVEL_ITEMS; ++k) {
        const int p = first + k * LEVEL_THREADS + threadIdx.x;
        y[k] = make_float2(0.f, 0.f);
        if (p < n) {
            const uint32_t slot = min((uint32_t)(words[p] & ((1ull << ks) - 1ull)), (uint32_t)n - 1u);
            perm[p] = slot;
            y[k] = Y[slot];
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < LEVEL_ITEMS; ++k) {
        const int p = first + k * LEVEL_THREADS + threadIdx.x;
        if (p < n) {
            Ys[p] = y[k];
            ax += (double)y[k].x; ay += (double)y[k].y;
            int tmin, tend;
            if constexpr (CT < 0) levels_at(kw, (uint32_t)n, (uint32_t)p, B, (uint32_t)C, &tmin, &tend);
            else levels_window<CT>(adjw + MARGIN + (p - first), B, C, &tmin, &tend);
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

// Per position: index of the first cell opened there, and the running sums of the sorted
// coordinates (ps[p] = sum of Ys[0..p), ps[n] = total).  Every workgroup first adds up the tile
// sums before its own tile (in a fixed order, so a run is reproducible; a few KB from the
// second-level cache instead of one more kernel); the last one also knows the number of cells.
__global__ __launch_bounds__(LEVEL_THREADS) void downsweep(const float2 *__restrict__ Ys,
                                                           const uint16_t *__restrict__ lev, int n,
                                                           const ScanPart *__restrict__ part,
                                                           uint32_t *__restrict__ cellseq, double2 *__restrict__ ps,
                                                           uint32_t *__restrict__ cell_p, uint8_t *__restrict__ cell_t,
                                                           uint32_t cap_cells, uint32_t *__restrict__ ncells,
                                                           uint32_t *status)
{
    __shared__ double wx[4], wy[4];
    __shared__ uint32_t wc[4];
    __shared__ double bx[4], by[4];
    __shared__ uint32_t bc[4];
    const int tid = threadIdx.x, w = tid >> 6;
    // tiles before this one
    double qx = 0.0, qy = 0.0;
    uint32_t qc = 0;
    for (int i = tid; i < (int)blockIdx.x; i += LEVEL_THREADS) {
        const ScanPart q = part[i];
        qx += q.sx; qy += q.sy; qc += q.cnt;
    }
    qx = wave_sum(qx); qy = wave_sum(qy); qc = wave_sum(qc);
    if (lane_id() == 0) { bx[w] = qx; by[w] = qy; bc[w] = qc; }
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
    double px = ((bx[0] + bx[1]) + bx[2]) + bx[3], py = ((by[0] + by[1]) + by[2]) + by[3];
    uint32_t pc = bc[0] + bc[1] + bc[2] + bc[3];
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
            if (p == n - 1) {
                cellseq[n] = pc;
                ps[n] = make_double2(px, py);
                *ncells = pc;
                if (pc > cap_cells) atomicOr(status, TSNE_STATUS_CELL_OVERFLOW);
            }
        }
    }
}

// First position in [s, e) whose digit (2 bits at sh) is >= q; e if none.
template <class Keys>
__device__ __forceinline__ uint32_t digit_lower_bound(const Keys &keys, uint32_t s, uint32_t e,
                                                      int sh, uint32_t q)
{
    while (s < e) {
        uint32_t mid = s + ((e - s) >> 1);
        if (((uint32_t)(keys[mid] >> sh) & 3u) < q) s = mid + 1; else e = mid;
    }
    return s;
}

// One lane per cell (cells are numbered in pre-order, so the cells of a workgroup start at
// non-decreasing positions and the keys they search sit in one stretch of CELL_WINDOW positions,
// staged in LDS).  A cell whose run of positions ends inside that stretch is finished on the spot,
// by searches that never leave LDS.  The large cells near the top of the tree would each be a
// chain of dozens of dependent memory reads in a single lane; they (and any cell that starts past
// the stretch) are put on a list instead and finished by write_big_cells, one wave per search.
constexpr int CELL_WINDOW = 2048;

// End of the cell (p, t) and the first positions of its children after the first; returns their number.
template <class Keys>
__device__ __forceinline__ int cell_extent(const Keys &keys, uint32_t lim, uint32_t n, uint32_t p, int t, int B, int C,
                                           uint64_t key, uint32_t *e_out, bool *leaf_out, uint32_t kid_pos[3])
{
    const uint32_t e = (t == 0) ? n : run_end(keys, lim, p, 2 * (B - t), key >> (2 * (B - t)));
    const bool leaf = e - p <= (uint32_t)C || t == B;
    int nk = 0;
    if (!leaf) {
        const int sh = 2 * (B - t - 1);
        uint32_t s = p;
        const uint32_t qfirst = (uint32_t)(key >> sh) & 3u;
        for (uint32_t q = qfirst + 1; q < 4; ++q) {
            const uint32_t b = digit_lower_bound(keys, s, e, sh, q);
            if (b < e && ((uint32_t)(keys[b] >> sh) & 3u) == q) kid_pos[nk++] = b;
            s = b;
        }
    }
    *e_out = e;
    *leaf_out = leaf;
    return nk;
}

__global__ __launch_bounds__(256) void write_cells(const uint64_t *__restrict__ words, int ks,
                                                   const uint32_t *__restrict__ cellseq,
                                                   const double2 *__restrict__ ps,
                                                   const uint32_t *__restrict__ cell_p, const uint8_t *__restrict__ cell_t,
                                                   const uint32_t *__restrict__ ncells, int n, int B, int C,
                                                   Cell *__restrict__ cells, uint32_t cap_cells,
                                                   uint32_t *__restrict__ big_count, uint2 *__restrict__ big_list,
                                                   uint32_t big_cap)
{
    __shared__ uint64_t kwin[CELL_WINDOW];
    const uint32_t m = min(*ncells, cap_cells);
    for (uint32_t base = blockIdx.x * 256u; base < m; base += gridDim.x * 256u) {
        const uint32_t id = base + threadIdx.x;
        const bool live = id < m;
        const uint32_t p_first = min(cell_p[base], (uint32_t)n - 1u);
        const uint32_t wlen = min((uint32_t)n - p_first, (uint32_t)CELL_WINDOW), wend = p_first + wlen;
        // the cell of this lane and the running sum at its first position: requested before the
        // window so that they travel together with it
        uint32_t p = 0;
        int t = 0;
        double2 s0 = make_double2(0.0, 0.0);
        if (live) { p = min(cell_p[id], (uint32_t)n - 1u); t = min((int)cell_t[id], B); s0 = ps[p]; }
        __syncthreads();                    // previous round's readers are done with the window
        for (uint32_t q = threadIdx.x; q < wlen; q += 256u) kwin[q] = words[p_first + q] >> ks;
        __syncthreads();
        if (!live) continue;
        const bool inside = p >= p_first && p < wend;
        const uint64_t key = inside ? kwin[p - p_first] : words[p] >> ks;
        // large: starts past the window, or shares its prefix with the window's last position
        // while the array goes on (the root, t = 0, shares it with every position)
        const bool big = !inside || (wend < (uint32_t)n &&
                                     (t == 0 || (kwin[wlen - 1] >> (2 * (B - t))) == (key >> (2 * (B - t)))));
        uint32_t e, kid_pos[3];
        bool leaf;
        int nk;
        if (big) {
            const uint32_t slot = atomicAdd(big_count, 1u);
            if (slot < big_cap) { big_list[slot] = make_uint2(p, (uint32_t)t); continue; }
            // list full (cannot happen for capacity n/8 + 1024 unless most cells are large): finish it here,
            // reading keys from memory wherever the window does not hold them
            KeyWindow kw;
            kw.words = words; kw.lds = kwin; kw.ks = ks; kw.lo = p_first; kw.len = wlen;
            nk = cell_extent(kw, (uint32_t)n, (uint32_t)n, p, t, B, C, key, &e, &leaf, kid_pos);
        } else {
            // the run ends before the window's last position (which is not part of it), or at n: no probe leaves LDS
            LdsKeys lk;
            lk.lds = kwin; lk.lo = p_first;
            nk = cell_extent(lk, wend < (uint32_t)n ? wend - 1u : (uint32_t)n, (uint32_t)n, p, t, B, C, key, &e, &leaf, kid_pos);
        }
        // the reads from memory that the searches lead to, together
        const double2 s1 = ps[e];
        const uint32_t cnt = e - p;
        Cell c;
        c.c1 = nk > 0 ? cellseq[kid_pos[0]] : TSNE_NONE;
        c.c2 = nk > 1 ? cellseq[kid_pos[1]] : TSNE_NONE;
        c.c3 = nk > 2 ? cellseq[kid_pos[2]] : TSNE_NONE;
        c.cx = (float)((s1.x - s0.x) / (double)cnt);
        c.cy = (float)((s1.y - s0.y) / (double)cnt);
        c.cnt = cnt;
        c.meta = (uint32_t)t | (leaf ? 0x100u : 0u);
        c.lo = p;
        cells[id] = c;
    }
}

// First position i in [lo, n) with (key[i] >> sh) >= target (n if there is none), found by the
// whole wave: every round the 64 lanes probe 64 evenly spaced positions of the remaining range,
// which shrinks 64-fold, so five rounds cover any n.  All lanes must call with the same
// arguments; every probed index lies inside [lo, n) whatever the keys hold.
__device__ __forceinline__ uint32_t wave_shifted_lower_bound(const uint64_t *__restrict__ words, int ks, uint32_t lo,
                                                             uint32_t n, int sh, uint64_t target)
{
    uint32_t hi = n;
    const uint32_t lane = (uint32_t)lane_id();
    while (lo < hi) {
        const uint32_t step = (hi - lo + 63u) >> 6;
        const uint64_t probe = (uint64_t)lo + (uint64_t)(lane + 1u) * step - 1ull;
        bool below = false;
        if (probe < (uint64_t)hi) below = ((words[probe] >> ks) >> sh) < target;
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
__global__ __launch_bounds__(256) void write_big_cells(const uint64_t *__restrict__ words, int ks,
                                                       const uint16_t *__restrict__ lev,
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
        const uint64_t key = words[p] >> ks;
        uint32_t found = (uint32_t)n;
        if (role == 0) {
            if (t > 0) {
                const int sh = 2 * (B - t);
                found = wave_shifted_lower_bound(words, ks, p, (uint32_t)n, sh, (key >> sh) + 1ull);
            }
        } else if (t < B) {
            const int sh = 2 * (B - t - 1);
            const uint64_t parent = t > 0 ? (key >> (2 * (B - t))) : 0ull;
            found = wave_shifted_lower_bound(words, ks, p, (uint32_t)n, sh, (parent << 2) + (uint64_t)role);
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
                    const uint32_t qfirst = (uint32_t)(key >> (2 * (B - t - 1))) & 3u;
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

// keys and spatial order in the caller's numbering
__global__ __launch_bounds__(256) void export_order_k(const uint64_t *__restrict__ words, int ks,
                                                      const uint32_t *__restrict__ orig, int n, uint64_t *__restrict__ keys_out,
                                                      int32_t *__restrict__ perm_out)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    const uint64_t w = words[p];
    const uint32_t o = orig[min((uint32_t)(w & ((1ull << ks) - 1ull)), (uint32_t)n - 1u)];
    if (keys_out) keys_out[min(o, (uint32_t)n - 1u)] = w >> ks;
    if (perm_out) perm_out[p] = (int32_t)o;
}

hipError_t launch_export_order(tsne_ctx *c, uint64_t *d_keys, int32_t *d_perm, hipStream_t s)
{
    const int n = c->p.n;
    hipLaunchKernelGGL(export_order_k, dim3((n + 255) / 256), dim3(256), 0, s, c->words[c->sorted_buf], c->key_shift,
                       c->orig[c->cur_state], n, d_keys, d_perm);
    return hipGetLastError();
}

// ------------------------------------------------------------------ host: enqueue the whole build
static int bbox_blocks(int n)
{
    int nb = (n + 255) / 256;
    return nb < BBOX_MAX_BLOCKS ? nb : BBOX_MAX_BLOCKS;
}

// Words per thread of the sort's tiles: a tile is a workgroup, and a launch is as long as its busiest compute unit,
// so the tile size is taken (from 8, 10 or 12 words a thread) to make the number of tiles per compute unit, rounded
// up, times the tile size smallest: 1,281,167 words are 313 tiles of 4096, which leaves 57 units with two, or 251
// tiles of 5120, one each.
int sort_items(int n, int num_cu)
{
    int best = 8;
    long long best_cost = -1;
    const int cu = num_cu > 0 ? num_cu : 256;
    for (int items = 8; items <= 12; items += 2) {
        const long long nblk = ((long long)n + SORT_THREADS * items - 1) / (SORT_THREADS * items);
        const long long cost = ((nblk + cu - 1) / cu) * items;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = items; }
    }
    return best;
}

template <int ITEMS>
static void sort_passes(tsne_ctx *c, int lo, int nbits, bool hist0, hipStream_t s)
{
    const int n = c->p.n;
    const int nblk = (n + SORT_THREADS * ITEMS - 1) / (SORT_THREADS * ITEMS);
    const int grid = 8 * ((nblk + 7) / 8);       // scatter_tile() deals the tiles to the XCDs
    int cur = 0;
    for (int plo = lo; plo < lo + nbits; plo += RADIX_BITS) {
        const int width = lo + nbits - plo < RADIX_BITS ? lo + nbits - plo : RADIX_BITS;
        const uint32_t mask = (1u << width) - 1u;
        if (!(hist0 && plo == lo))
            hipLaunchKernelGGL(radix_hist<ITEMS>, dim3(nblk), dim3(SORT_THREADS), 0, s, c->words[cur], n, plo, mask, c->hist,
                               nblk);
        hipLaunchKernelGGL(radix_scan, dim3(RADIX / SCAN_DIGITS), dim3(SCAN_DIGITS * SCAN_SEGS), 0, s, c->hist, nblk,
                           c->dtot);
        hipLaunchKernelGGL(radix_scatter<ITEMS>, dim3(grid), dim3(SORT_THREADS), 0, s, c->words[cur], c->words[cur ^ 1], n,
                           plo, mask, c->hist, c->dtot, nblk);
        cur ^= 1;
    }
    c->sorted_buf = cur;
}

// Stable LSD radix sort of words[0] on bits [lo, lo + nbits), RADIX_BITS a pass.
hipError_t launch_sort(tsne_ctx *c, int lo, int nbits, bool hist0, hipStream_t s)
{
    switch (c->sort_items) {
    case 10: sort_passes<10>(c, lo, nbits, hist0, s); break;
    case 12: sort_passes<12>(c, lo, nbits, hist0, s); break;
    default: sort_passes<8>(c, lo, nbits, hist0, s); break;
    }
    return hipGetLastError();
}

hipError_t launch_unpack_perm(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n;
    hipLaunchKernelGGL(unpack_perm_k, dim3((n + 255) / 256), dim3(256), 0, s, c->words[c->sorted_buf], n, c->perm);
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

// Step 1 second half on its own, for a step whose attraction wants the root square before the sort is enqueued.
hipError_t launch_tree_root(tsne_ctx *c, hipStream_t s)
{
    if (c->p.n <= SMALL_SORT_MAX) return hipSuccess;      // (there the root comes out of the one launch that also sorts)
    hipLaunchKernelGGL(bbox_final, dim3(1), dim3(c->bbox_nparts > 1024 ? 1024 : 256), 0, s, c->bbox_part, c->bbox_nparts,
                       c->p.morton_bits, c->root, c->status);
    c->root_fresh = 1;
    return hipGetLastError();
}

// Step 1 second half, step 2a and step 4: root square, keys, spatial sort.
hipError_t launch_tree_sort(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n, B = c->p.morton_bits, ks = c->key_shift;
    const float2 *Y = c->Yi;
    if (n <= SMALL_SORT_MAX) {
        int m = 512;
        while (m < n) m <<= 1;
        hipLaunchKernelGGL(small_root_keys_sort<3>, dim3(1), dim3(m >> 3), small_sort_lds(m), s, Y, n, m, c->bbox_part,
                           c->bbox_nparts, B, ks, c->root, c->words[0], c->status);
        c->sorted_buf = 0;
        return hipGetLastError();
    }
    if (!c->root_fresh)
        hipLaunchKernelGGL(bbox_final, dim3(1), dim3(c->bbox_nparts > 1024 ? 1024 : 256), 0, s, c->bbox_part, c->bbox_nparts, B,
                           c->root, c->status);
    c->root_fresh = 0;
    const int items = c->sort_items, nblk = (n + SORT_THREADS * items - 1) / (SORT_THREADS * items);
    const int width0 = 2 * B < RADIX_BITS ? 2 * B : RADIX_BITS;
    if (items == 10)
        hipLaunchKernelGGL(morton_encode_hist<10>, dim3(nblk), dim3(SORT_THREADS), 0, s, Y, n, c->root, B, ks,
                           (1u << width0) - 1u, c->words[0], c->hist, nblk);
    else if (items == 12)
        hipLaunchKernelGGL(morton_encode_hist<12>, dim3(nblk), dim3(SORT_THREADS), 0, s, Y, n, c->root, B, ks,
                           (1u << width0) - 1u, c->words[0], c->hist, nblk);
    else
        hipLaunchKernelGGL(morton_encode_hist<8>, dim3(nblk), dim3(SORT_THREADS), 0, s, Y, n, c->root, B, ks,
                           (1u << width0) - 1u, c->words[0], c->hist, nblk);
    return launch_sort(c, ks, 2 * B, true, s);
}

// Steps 2b, 2c and 3: cells, counts, centres of mass from the sorted keys.
hipError_t launch_tree_cells(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n, B = c->p.morton_bits, C = c->p.leaf_cap, ks = c->key_shift;
    const float2 *Y = c->Yi;
    const int nb = (n + 255) / 256;
    const uint64_t *words = c->words[c->sorted_buf];
    int nl = (n + LEVEL_TILE - 1) / LEVEL_TILE;
    if (C == 8)
        hipLaunchKernelGGL(gather_levels<8>, dim3(nl), dim3(LEVEL_THREADS), 0, s, Y, words, ks, n, B, C, c->Ys, c->perm,
                           c->lev, c->part, c->big_count);
    else if (C <= LEVELS_WINDOW_MAXC)
        hipLaunchKernelGGL(gather_levels<0>, dim3(nl), dim3(LEVEL_THREADS), 0, s, Y, words, ks, n, B, C, c->Ys, c->perm,
                           c->lev, c->part, c->big_count);
    else
        hipLaunchKernelGGL(gather_levels<-1>, dim3(nl), dim3(LEVEL_THREADS), 0, s, Y, words, ks, n, B, C, c->Ys, c->perm,
                           c->lev, c->part, c->big_count);
    hipLaunchKernelGGL(downsweep, dim3(nl), dim3(LEVEL_THREADS), 0, s, c->Ys, c->lev, n, c->part, c->cellseq, c->ps,
                       c->cell_p, c->cell_t, (uint32_t)c->cap_cells, c->ncells, c->status);
    // grid sized for n / 2 cells (a typical tree has about n / 3); the kernel strides if there are more
    hipLaunchKernelGGL(write_cells, dim3((nb + 1) / 2), dim3(256), 0, s, words, ks, c->cellseq, c->ps, c->cell_p, c->cell_t,
                       c->ncells, n, B, C, c->cells, (uint32_t)c->cap_cells, c->big_count, c->big_list,
                       (uint32_t)c->big_cap);
    hipLaunchKernelGGL(write_big_cells, dim3(4096), dim3(256), 0, s, words, ks, c->lev,
                       c->cellseq, c->ps, n, B, C, c->cells, (uint32_t)c->cap_cells, c->big_count, c->big_list,
                       (uint32_t)c->big_cap);
    return hipGetLastError();
}
