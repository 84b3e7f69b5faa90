// Renumbering of the points.
//
// The paper names the attractive forces as the bottleneck because the sparsity pattern of P is
// disorganised (Sec. IV-D): row i gathers y_j from all over memory.  The library therefore keeps
// its own numbering of the points ("slots", `orig` maps them back to the caller's indices) in
// which neighbours in P get nearby numbers -- from the structure of P (below) or from the
// spatial order of the embedding, which the tree build computes anyway (Sec. III-C step 4).
// In that numbering almost all of P lies in a band around the diagonal.  The private copy of
// P is stored split: the near part (|column - row| <= ATTRACT_BAND), which the attraction
// kernel serves from a sliding window of Y in LDS, and the far remainder.  Values and the
// order of the entries inside each part of a row are those of the caller's P.
#include "tsne_internal.h"

#include <algorithm>

// position p of the new order takes over old slot s = perm[p]
__global__ __launch_bounds__(256) void reorder_state_k(const uint32_t *__restrict__ perm, int n,
                                                       const uint32_t *__restrict__ orig_in, uint32_t *__restrict__ orig_out,
                                                       const float2 *__restrict__ u_in, float2 *__restrict__ u_out,
                                                       const float2 *__restrict__ g_in, float2 *__restrict__ g_out,
                                                       uint32_t *__restrict__ inv)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    const uint32_t s = min(perm[p], (uint32_t)n - 1u);
    const uint32_t o = min(orig_in[s], (uint32_t)n - 1u);
    orig_out[p] = o;
    u_out[p] = u_in[s];
    g_out[p] = g_in[s];
    inv[o] = (uint32_t)p;
}

__global__ void zero_word_k(uint32_t *w) { *w = 0u; }

__device__ __forceinline__ bool in_band(uint32_t col_slot, int row_slot)
{
    const int d = (int)col_slot - row_slot;
    return d <= ATTRACT_BAND && d >= -ATTRACT_BAND;
}

// 16 lanes per slot p: how many entries of the caller's row orig[p] fall in the band
__global__ __launch_bounds__(256) void split_count_k(const uint32_t *__restrict__ orig, const uint32_t *__restrict__ inv,
                                                     int n, const int32_t *__restrict__ urp,
                                                     const int32_t *__restrict__ ucol, int32_t *__restrict__ len_near,
                                                     int32_t *__restrict__ len_far, uint32_t *__restrict__ far_rows,
                                                     uint32_t *__restrict__ far_count)
{
    const int p = (int)((blockIdx.x * 256u + threadIdx.x) / 16);
    const int sub = (int)(threadIdx.x % 16);
    int near = 0, len = 0;
    if (p < n) {
        const uint32_t u = min(orig[p], (uint32_t)n - 1u);
        const int src = urp[u];
        len = urp[u + 1] - src;
        for (int e = sub; e < len; e += 16)
            near += in_band(inv[min((uint32_t)ucol[src + e], (uint32_t)n - 1u)], p) ? 1 : 0;
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) near += __shfl_xor(near, o, WAVE);
    if (p < n && sub == 0) {
        len_near[p] = (near + ATTRACT_CHUNK - 1) / ATTRACT_CHUNK * ATTRACT_CHUNK;     // padded to whole chunks
        len_far[p] = len - near;
        if (len > near) far_rows[atomicAdd(far_count, 1u)] = (uint32_t)p;   // any order will do
    }
}

// rp_out = base + exclusive prefix sum of len (single block; runs once per renumbering)
__global__ __launch_bounds__(1024) void scan_len_k(const int32_t *__restrict__ len, int n, const int32_t *__restrict__ base,
                                                   int32_t *__restrict__ rp_out)
{
    __shared__ long long ws[16];
    const int per = (n + 1023) / 1024;
    const int s = threadIdx.x * per, e = min(n, s + per);
    long long a = 0;
    for (int i = s; i < e; ++i) a += len[i];
    long long inc = a;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        long long t = __shfl_up(inc, o, WAVE);
        if (lane_id() >= o) inc += t;
    }
    if (lane_id() == WAVE - 1) ws[threadIdx.x >> 6] = inc;
    __syncthreads();
    long long pre = inc - a + (base ? (long long)*base : 0ll);
    for (int q = 0; q < (int)(threadIdx.x >> 6); ++q) pre += ws[q];
    for (int i = s; i < e; ++i) { rp_out[i] = (int32_t)pre; pre += len[i]; }
    if (threadIdx.x == 1023) rp_out[n] = (int32_t)pre;
}

// 16 lanes copy one row: columns are relabelled, the entries go to the near or the far part in
// their original order, and the near part is filled up to whole chunks with (own slot, 0)
__global__ __launch_bounds__(256) void split_fill_k(const uint32_t *__restrict__ orig, const uint32_t *__restrict__ inv,
                                                    int n, const int32_t *__restrict__ urp,
                                                    const int32_t *__restrict__ ucol, const float *__restrict__ uval,
                                                    const int32_t *__restrict__ rp_near, const int32_t *__restrict__ rp_far,
                                                    uint16_t *__restrict__ col_near, int32_t *__restrict__ col_far,
                                                    float *__restrict__ val_s)
{
    const int p = (int)((blockIdx.x * 256u + threadIdx.x) / 16);
    const int sub = (int)(threadIdx.x % 16);
    if (p >= n) return;
    const int shift = (int)(lane_id() & 48);          // first lane of this 16-lane group
    const uint32_t below = (1u << sub) - 1u;
    const uint32_t u = min(orig[p], (uint32_t)n - 1u);
    const int src = urp[u], len = urp[u + 1] - src;
    int dn = rp_near[p], df = rp_far[p];
    const int far0 = rp_far[0];
    const int end_near = rp_near[p + 1];
    for (int e0 = 0; e0 < len; e0 += 16) {
        const int e = e0 + sub;
        const bool in = e < len;
        uint32_t cs = 0u;
        float v = 0.f;
        if (in) {
            cs = inv[min((uint32_t)ucol[src + e], (uint32_t)n - 1u)];
            v = uval[src + e];
        }
        const bool near = in && in_band(cs, p);
        const uint32_t mn = (uint32_t)(__ballot(near) >> shift) & 0xFFFFu;
        const uint32_t mf = (uint32_t)(__ballot(in && !near) >> shift) & 0xFFFFu;
        if (near) {   // near columns are stored as the byte offset of the point in the ring of Y
            const int d = dn + __popc(mn & below);
            col_near[d] = (uint16_t)((cs % (uint32_t)ATTRACT_RING) * 8u);
            val_s[d] = v;
        } else if (in) {
            const int d = df + __popc(mf & below);
            col_far[d - far0] = (int32_t)cs;
            val_s[d] = v;
        }
        dn += __popc(mn);
        df += __popc(mf);
    }
    for (int d = dn + sub; d < end_near; d += 16) {       // padding: own point, weight 0
        col_near[d] = (uint16_t)((p % ATTRACT_RING) * 8);
        val_s[d] = 0.f;
    }
}


// ---- the far part once more, bucketed by tiles (for attract_far_tiled)
// meta: [0] tiles in use, [1] largest value of P (bits of a non-negative float), [2] longest far row.
__global__ void ft_begin_k(uint32_t *meta) { meta[0] = 0u; meta[1] = 0u; meta[2] = 0u; }

__global__ __launch_bounds__(256) void ft_stats_k(const float *__restrict__ uval, int64_t nnz,
                                                  const int32_t *__restrict__ len_far, int n, uint32_t *meta)
{
    uint32_t pm = 0u, lm = 0u;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < nnz; e += stride) {
        const float v = uval[e];
        if (v > 0.f) pm = max(pm, __float_as_uint(v));
    }
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) lm = max(lm, (uint32_t)len_far[i]);
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) {
        pm = max(pm, (uint32_t)__shfl_xor((int)pm, o, WAVE));
        lm = max(lm, (uint32_t)__shfl_xor((int)lm, o, WAVE));
    }
    if (lane_id() == 0) {
        if (pm) atomicMax(meta + 1, pm);
        if (lm) atomicMax(meta + 2, lm);
    }
}

// mode: 0 = tiles if the far part is at least half of the entries and there are at least FT_MIN_POINTS points
// (measured on four 50-dimensional blobs: 0.23 against 0.30 ms per iteration row by row at 128,000 points, 0.57
// against 0.47 at 256,000: below the limit all of Y stays in the second-level cache; a far part
// that is a minority -- clusters a little wider than the band -- is quicker row by row beside the tree
// build: measured on the 400,000-point, 200-cluster workload), 1 = never, 2 = always
__global__ void ft_decide_k(const int32_t *__restrict__ rp_far, int n, int64_t nnz, int mode, uint32_t *meta)
{
    const int64_t far_total = (int64_t)rp_far[n] - rp_far[0];
    meta[0] = far_total > 0 && (mode == 2 || (mode == 0 && far_total * 2 >= nnz && n >= FT_MIN_POINTS)) ? 1u : 0u;
    meta[4] = (uint32_t)far_total;      // for the host: how many workgroups the tile kernel is worth
}

__global__ __launch_bounds__(256) void ft_zero_k(uint32_t *__restrict__ cnt, int64_t tiles, const uint32_t *meta)
{
    if (!meta[0]) return;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < tiles; t += stride) cnt[t] = 0u;
}

// 16 lanes per row; FILL: place the entries (the counts of ft_count run down to 0 as positions are handed out)
template <bool FILL>
__global__ __launch_bounds__(256) void ft_scatter_k(const int32_t *__restrict__ rp_far, const int32_t *__restrict__ col_far,
                                                    const float *__restrict__ val_s, int n, int nct,
                                                    uint32_t *__restrict__ cnt, const int32_t *__restrict__ ptr,
                                                    int32_t *__restrict__ tcol, uint16_t *__restrict__ trow,
                                                    float *__restrict__ tval, const uint32_t *meta)
{
    if (!meta[0]) return;
    const int p = (int)((blockIdx.x * 256u + threadIdx.x) / 16);
    const int sub = (int)(threadIdx.x % 16);
    if (p >= n) return;
    const int far0 = rp_far[0];
    const int64_t tile0 = (int64_t)(p / FT_ROWS) * nct;
    for (int e = rp_far[p] + sub; e < rp_far[p + 1]; e += 16) {
        const uint32_t cs = min((uint32_t)col_far[e - far0], (uint32_t)n - 1u);
        const int64_t t = tile0 + cs / FT_COLS;
        if (!FILL) atomicAdd(cnt + t, 1u);
        else {
            const uint32_t left = atomicSub(cnt + t, 1u);      // any order inside the tile
            const int pos = ptr[t] + (int)left - 1;
            tcol[pos] = (int32_t)cs;
            trow[pos] = (uint16_t)(p % FT_ROWS);
            tval[pos] = val_s[e];
        }
    }
}

// The entries of every tile, placed in any order, into the order of their columns, FT_SORT_PIECE entries
// at a time (a counting sort in LDS over the tile's FT_COLS columns).  A gather instruction pays per cache
// line of Y that its 64 lanes touch: 64 consecutive entries of a sorted piece of m entries span about
// 64 / m of the tile's 128 lines instead of some 50 of them.  The row sums do not depend on the order.
constexpr int FT_SORT_PIECE = 4096;
__global__ __launch_bounds__(256) void ft_sort_k(const int32_t *__restrict__ ptr, int64_t tiles, int nct,
                                                 int32_t *__restrict__ tcol, uint16_t *__restrict__ trow,
                                                 float *__restrict__ tval, const uint32_t *meta)
{
    if (!meta[0]) return;
    __shared__ int32_t scol[FT_SORT_PIECE];
    __shared__ float sval[FT_SORT_PIECE];
    __shared__ uint16_t srow[FT_SORT_PIECE];
    __shared__ uint32_t bin[FT_COLS];
    __shared__ uint32_t wsum[4];
    static_assert(FT_COLS % 256 == 0, "columns per thread");
    constexpr int BPT = FT_COLS / 256;
    const int tid = (int)threadIdx.x, w = tid >> 6;
    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        const int b0 = ptr[t], b1 = ptr[t + 1];
        const uint32_t c0 = (uint32_t)(t % nct) * (uint32_t)FT_COLS;
        for (int s0 = b0; s0 < b1; s0 += FT_SORT_PIECE) {     // (b0, b1: the same for every thread)
            const int m = min(FT_SORT_PIECE, b1 - s0);
            __syncthreads();                                  // the previous piece is written out
            for (int i = tid; i < FT_COLS; i += 256) bin[i] = 0u;
            __syncthreads();
            for (int i = tid; i < m; i += 256) {
                const int32_t cj = tcol[s0 + i];
                scol[i] = cj;
                srow[i] = trow[s0 + i];
                sval[i] = tval[s0 + i];
                atomicAdd(&bin[min((uint32_t)cj - c0, (uint32_t)FT_COLS - 1u)], 1u);
            }
            __syncthreads();
            uint32_t loc[BPT], sum = 0;
#pragma unroll
            for (int k = 0; k < BPT; ++k) { loc[k] = bin[tid * BPT + k]; sum += loc[k]; }
            int tot;
            const int ex = wave_excl_scan((int)sum, &tot);
            if (lane_id() == 0) wsum[w] = (uint32_t)tot;
            __syncthreads();
            uint32_t run = (uint32_t)ex;
            for (int k = 0; k < w; ++k) run += wsum[k];
#pragma unroll
            for (int k = 0; k < BPT; ++k) { bin[tid * BPT + k] = run; run += loc[k]; }
            __syncthreads();
            for (int i = tid; i < m; i += 256) {
                const int32_t cj = scol[i];
                const uint32_t pos = min(atomicAdd(&bin[min((uint32_t)cj - c0, (uint32_t)FT_COLS - 1u)], 1u), (uint32_t)m - 1u);
                tcol[s0 + pos] = cj;
                trow[s0 + pos] = srow[i];
                tval[s0 + pos] = sval[i];
            }
        }
    }
}

hipError_t launch_reorder(tsne_ctx *c, hipStream_t s, int tiles_mode)
{
    const int n = c->p.n;
    const uint32_t *perm = c->perm;
    const int a = c->cur_state, b = a ^ 1;
    hipLaunchKernelGGL(reorder_state_k, dim3((n + 255) / 256), dim3(256), 0, s, perm, n, c->orig[a], c->orig[b],
                       c->uYb[a], c->uYb[b], c->gainsb[a], c->gainsb[b], c->inv);
    const unsigned blocks = (unsigned)(((int64_t)n * 16 + 255) / 256);
    hipLaunchKernelGGL(zero_word_k, dim3(1), dim3(1), 0, s, c->far_count);
    hipLaunchKernelGGL(split_count_k, dim3(blocks), dim3(256), 0, s, c->orig[b], c->inv, n, c->user_row_ptr, c->user_col,
                       c->len_near, c->len_far, c->far_rows, c->far_count);
    hipLaunchKernelGGL(scan_len_k, dim3(1), dim3(1024), 0, s, c->len_near, n, (const int32_t *)nullptr, c->rp_near);
    hipLaunchKernelGGL(scan_len_k, dim3(1), dim3(1024), 0, s, c->len_far, n, (const int32_t *)(c->rp_near + n), c->rp_far);
    hipLaunchKernelGGL(split_fill_k, dim3(blocks), dim3(256), 0, s, c->orig[b], c->inv, n, c->user_row_ptr, c->user_col,
                       c->user_val, c->rp_near, c->rp_far, c->col_near, c->col_far, c->val_s);
    if (c->ft_tiles > 0) {
        const unsigned sblocks = (unsigned)std::min<int64_t>(4096, (std::max<int64_t>(c->nnz, n) + 255) / 256);
        const unsigned zblocks = (unsigned)std::min<int64_t>(4096, (c->ft_tiles + 255) / 256);
        hipLaunchKernelGGL(ft_begin_k, dim3(1), dim3(1), 0, s, c->ft_meta);
        hipLaunchKernelGGL(ft_stats_k, dim3(sblocks), dim3(256), 0, s, c->user_val, c->nnz, c->len_far, n, c->ft_meta);
        hipLaunchKernelGGL(ft_decide_k, dim3(1), dim3(1), 0, s, c->rp_far, n, c->nnz, tiles_mode, c->ft_meta);
        hipLaunchKernelGGL(ft_zero_k, dim3(zblocks), dim3(256), 0, s, c->ft_cnt, c->ft_tiles, c->ft_meta);
        hipLaunchKernelGGL(ft_scatter_k<false>, dim3(blocks), dim3(256), 0, s, c->rp_far, c->col_far, c->val_s, n, c->ft_nct,
                           c->ft_cnt, c->ft_ptr, c->ft_col, c->ft_row, c->ft_val, c->ft_meta);
        hipLaunchKernelGGL(scan_len_k, dim3(1), dim3(1024), 0, s, (const int32_t *)c->ft_cnt, (int)c->ft_tiles,
                           (const int32_t *)nullptr, c->ft_ptr);
        hipLaunchKernelGGL(ft_scatter_k<true>, dim3(blocks), dim3(256), 0, s, c->rp_far, c->col_far, c->val_s, n, c->ft_nct,
                           c->ft_cnt, c->ft_ptr, c->ft_col, c->ft_row, c->ft_val, c->ft_meta);
        hipLaunchKernelGGL(ft_sort_k, dim3((unsigned)std::min<int64_t>(c->ft_tiles, 1 << 20)), dim3(256), 0, s, c->ft_ptr,
                           c->ft_tiles, c->ft_nct, c->ft_col, c->ft_row, c->ft_val, c->ft_meta);
    }
    hipError_t e = launch_iota(c->row_order, n, s);
    if (e != hipSuccess) return e;
    c->cur_state = b;
    c->arow_valid = 0;
    c->identity = 0;
    return hipGetLastError();
}

// ---- ordering of the points by the structure of P alone
// x_i starts as a hash of i in [0,1) and is replaced T times by the p-weighted mean of x over
// row i of P.  Values inside a well-connected neighbourhood converge to a common value long
// before different neighbourhoods mix, so sorting by x groups the points the way P links them.
__device__ __forceinline__ uint32_t mix32(uint32_t v)
{
    v ^= v >> 16; v *= 0x7feb352du; v ^= v >> 15; v *= 0x846ca68bu; v ^= v >> 16;
    return v;
}

__global__ __launch_bounds__(256) void graph_seed_k(float *__restrict__ x, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) x[i] = (float)(mix32((uint32_t)i + 0x9e3779b9u) >> 8) * (1.0f / 16777216.0f);
}

__global__ __launch_bounds__(256) void graph_smooth_k(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col,
                                                      const float *__restrict__ val, const float *__restrict__ x, int n,
                                                      float *__restrict__ xo)
{
    const int row = (int)((blockIdx.x * 256u + threadIdx.x) / 16);
    const int sub = (int)(threadIdx.x % 16);
    float a = 0.f, w = 0.f;
    if (row < n) {
        const int s = row_ptr[row], e = row_ptr[row + 1];
        for (int j0 = s + sub; j0 < e; j0 += 64) {      // four entries per lane in flight
            float v[4], xv[4];
            int cj[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = j0 + 16 * q;
                v[q] = j < e ? val[j] : 0.f;
                cj[q] = j < e ? col[j] : row;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) xv[q] = x[min((uint32_t)cj[q], (uint32_t)n - 1u)];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                a = fmaf(v[q], xv[q], a);
                w += v[q];
            }
        }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) { a += __shfl_xor(a, o, WAVE); w += __shfl_xor(w, o, WAVE); }
    if (row < n && sub == 0) xo[row] = w > 0.f ? a / w : x[row];
}

__global__ __launch_bounds__(256) void graph_keys_k(const float *__restrict__ x, int n, uint64_t *__restrict__ words)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t u = __float_as_uint(x[i]);     // x >= 0: the bit pattern is already ordered
    words[i] = ((uint64_t)u << 32) | (uint32_t)i;
}

hipError_t launch_graph_order(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n;
    float *xa = (float *)c->Yi, *xb = xa + n;      // Yi (2n floats) is free between steps
    hipLaunchKernelGGL(graph_seed_k, dim3((n + 255) / 256), dim3(256), 0, s, xa, n);
    const unsigned blocks = (unsigned)(((int64_t)n * 16 + 255) / 256);
    for (int t = 0; t < c->p.graph_order_iters; ++t) {
        hipLaunchKernelGGL(graph_smooth_k, dim3(blocks), dim3(256), 0, s, c->user_row_ptr, c->user_col, c->user_val, xa, n, xb);
        float *tmp = xa; xa = xb; xb = tmp;
    }
    hipLaunchKernelGGL(graph_keys_k, dim3((n + 255) / 256), dim3(256), 0, s, xa, n, c->words[0]);
    hipError_t e = launch_sort(c, 32, 32, false, s);
    return e != hipSuccess ? e : launch_unpack_perm(c, s);
}

// out[orig[s]] = in[s] and its inverse (copies between slot order and the caller's order)
__global__ __launch_bounds__(256) void scatter2_k(const float2 *__restrict__ in, const uint32_t *__restrict__ orig,
                                                  float2 *__restrict__ out, int n)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < n) out[min(orig[s], (uint32_t)n - 1u)] = in[s];
}

__global__ __launch_bounds__(256) void gather2_k(const float2 *__restrict__ in, const uint32_t *__restrict__ orig,
                                                 float2 *__restrict__ out, int n)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s < n) out[s] = in[min(orig[s], (uint32_t)n - 1u)];
}

hipError_t launch_scatter2(const float2 *in, const uint32_t *orig, float2 *out, int n, hipStream_t s)
{
    hipLaunchKernelGGL(scatter2_k, dim3((n + 255) / 256), dim3(256), 0, s, in, orig, out, n);
    return hipGetLastError();
}

hipError_t launch_gather2(const float2 *in, const uint32_t *orig, float2 *out, int n, hipStream_t s)
{
    hipLaunchKernelGGL(gather2_k, dim3((n + 255) / 256), dim3(256), 0, s, in, orig, out, n);
    return hipGetLastError();
}
