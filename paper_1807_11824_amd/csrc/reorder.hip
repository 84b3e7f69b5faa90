// Renumbering of the points along the current spatial order.
//
// The paper names the attractive forces as the bottleneck because the sparsity pattern of P is
// disorganised (Sec. IV-D): row i gathers y_j from all over memory.  Once the embedding has
// formed, neighbours in P are neighbours in the plane, so storing the points in the order of
// the space-filling curve (which the tree build computes anyway, Sec. III-C step 4) turns those
// gathers into accesses to a small, cache-resident window.  Nothing the method computes
// changes: P keeps its values and the order of the entries inside every row, only row and
// column numbers are relabelled; `orig` maps the library's slots back to the caller's indices.
#include "tsne_internal.h"

// position p of the new order takes over old slot s = perm[p]
__global__ __launch_bounds__(256) void reorder_state_k(const uint32_t *__restrict__ perm, int n,
                                                       const uint32_t *__restrict__ orig_in, uint32_t *__restrict__ orig_out,
                                                       const float2 *__restrict__ u_in, float2 *__restrict__ u_out,
                                                       const float2 *__restrict__ g_in, float2 *__restrict__ g_out,
                                                       const int32_t *__restrict__ rp_in, uint32_t *__restrict__ inv,
                                                       int32_t *__restrict__ len)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    const uint32_t s = min(perm[p], (uint32_t)n - 1u);
    orig_out[p] = orig_in[s];
    u_out[p] = u_in[s];
    g_out[p] = g_in[s];
    inv[s] = (uint32_t)p;
    len[p] = rp_in[s + 1] - rp_in[s];
}

// rp_out = exclusive prefix sum of len (single block; runs once per renumbering)
__global__ __launch_bounds__(1024) void scan_len_k(const int32_t *__restrict__ len, int n, int32_t *__restrict__ rp_out)
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
    long long pre = inc - a;
    for (int q = 0; q < (int)(threadIdx.x >> 6); ++q) pre += ws[q];
    for (int i = s; i < e; ++i) { rp_out[i] = (int32_t)pre; pre += len[i]; }
    if (threadIdx.x == 1023) rp_out[n] = (int32_t)pre;
}

// 16 lanes copy one row: entries keep their order, columns are relabelled
__global__ __launch_bounds__(256) void reorder_rows_k(const uint32_t *__restrict__ perm, const uint32_t *__restrict__ inv,
                                                      int n, const int32_t *__restrict__ rp_in,
                                                      const int32_t *__restrict__ col_in, const float *__restrict__ val_in,
                                                      const int32_t *__restrict__ rp_out, int32_t *__restrict__ col_out,
                                                      float *__restrict__ val_out)
{
    const int p = (int)((blockIdx.x * 256u + threadIdx.x) / 16);
    const int sub = (int)(threadIdx.x % 16);
    if (p >= n) return;
    const uint32_t s = min(perm[p], (uint32_t)n - 1u);
    const int src = rp_in[s], len = rp_in[s + 1] - src, dst = rp_out[p];
    for (int e = sub; e < len; e += 16) {
        col_out[dst + e] = (int32_t)inv[min((uint32_t)col_in[src + e], (uint32_t)n - 1u)];
        val_out[dst + e] = val_in[src + e];
    }
}

hipError_t launch_reorder(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n;
    const uint32_t *perm = c->idx[c->sorted_buf];
    const int a = c->cur_state, b = a ^ 1;
    const int pb = c->cur_P ^ 1;        // internal CSR buffer to fill
    hipLaunchKernelGGL(reorder_state_k, dim3((n + 255) / 256), dim3(256), 0, s, perm, n, c->orig[a], c->orig[b],
                       c->uYb[a], c->uYb[b], c->gainsb[a], c->gainsb[b], c->row_ptr, c->inv, c->lenbuf);
    hipLaunchKernelGGL(scan_len_k, dim3(1), dim3(1024), 0, s, c->lenbuf, n, c->rp_i[pb]);
    const unsigned blocks = (unsigned)(((int64_t)n * 16 + 255) / 256);
    hipLaunchKernelGGL(reorder_rows_k, dim3(blocks), dim3(256), 0, s, perm, c->inv, n, c->row_ptr, c->col, c->val,
                       c->rp_i[pb], c->col_i[pb], c->val_i[pb]);
    hipError_t e = launch_iota(c->row_order, n, s);
    if (e != hipSuccess) return e;
    c->cur_state = b;
    c->cur_P = pb;
    c->row_ptr = c->rp_i[pb]; c->col = c->col_i[pb]; c->val = c->val_i[pb];
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
        for (int j = s + sub; j < e; j += 16) {
            const float v = val[j];
            a = fmaf(v, x[min((uint32_t)col[j], (uint32_t)n - 1u)], a);
            w += v;
        }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) { a += __shfl_xor(a, o, WAVE); w += __shfl_xor(w, o, WAVE); }
    if (row < n && sub == 0) xo[row] = w > 0.f ? a / w : x[row];
}

__global__ __launch_bounds__(256) void graph_keys_k(const float *__restrict__ x, int n, uint32_t *__restrict__ keys,
                                                    uint32_t *__restrict__ idx)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t u = __float_as_uint(x[i]);     // x >= 0: the bit pattern is already ordered
    keys[i] = u;
    idx[i] = (uint32_t)i;
}

hipError_t launch_graph_order(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n;
    float *xa = (float *)c->Yi, *xb = xa + n;      // Yi (2n floats) is free between steps
    hipLaunchKernelGGL(graph_seed_k, dim3((n + 255) / 256), dim3(256), 0, s, xa, n);
    const unsigned blocks = (unsigned)(((int64_t)n * 16 + 255) / 256);
    for (int t = 0; t < c->p.graph_order_iters; ++t) {
        hipLaunchKernelGGL(graph_smooth_k, dim3(blocks), dim3(256), 0, s, c->row_ptr, c->col, c->val, xa, n, xb);
        float *tmp = xa; xa = xb; xb = tmp;
    }
    hipLaunchKernelGGL(graph_keys_k, dim3((n + 255) / 256), dim3(256), 0, s, xa, n, c->keys[0], c->idx[0]);
    return launch_sort(c, 32, s);
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

// keys and spatial order in the caller's numbering (tests only)
__global__ __launch_bounds__(256) void export_order_k(const uint32_t *__restrict__ keys_slot, const uint32_t *__restrict__ perm,
                                                      const uint32_t *__restrict__ orig, int n, uint32_t *__restrict__ keys_out,
                                                      int32_t *__restrict__ perm_out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (keys_out) keys_out[min(orig[i], (uint32_t)n - 1u)] = keys_slot[i];
    if (perm_out) perm_out[i] = (int32_t)orig[min(perm[i], (uint32_t)n - 1u)];
}

hipError_t launch_export_order(tsne_ctx *c, uint32_t *d_keys, int32_t *d_perm, hipStream_t s)
{
    const int n = c->p.n;
    hipLaunchKernelGGL(export_order_k, dim3((n + 255) / 256), dim3(256), 0, s, c->keys_orig, c->idx[c->sorted_buf],
                       c->orig[c->cur_state], n, d_keys, d_perm);
    return hipGetLastError();
}
