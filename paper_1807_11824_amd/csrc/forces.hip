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

// Variant for renumbered points (slot order follows the structure of P, so row i's columns lie
// mostly within a band around i): a workgroup owns ROWS consecutive rows and first stages
// Y[r0 - HALO, r0 + ROWS + HALO) in LDS; gathers that fall inside the window are LDS reads, the
// rest go to memory as before.  Entries of a row are taken in the same lane order as in the
// kernel above, so both produce the same sums.
#ifndef AW_HALO_N
#define AW_HALO_N 1280
#endif
#ifndef AW_ROWS_N
#define AW_ROWS_N 128
#endif
#ifndef AW_DUAL_N
#define AW_DUAL_N 2
#endif
constexpr int AW_ROWS = AW_ROWS_N, AW_HALO = AW_HALO_N, AW_LPR = 16, AW_U = 4, AW_DUAL = AW_DUAL_N;

__global__ __launch_bounds__(256) void attract_csr_window(const int32_t *__restrict__ row_ptr,
                                                          const int32_t *__restrict__ col, const float *__restrict__ val,
                                                          const float2 *__restrict__ Y, int n, float2 *__restrict__ A)
{
    constexpr int WIN = AW_ROWS + 2 * AW_HALO;
    __shared__ float2 win[WIN];
    const int r0 = (int)blockIdx.x * AW_ROWS;
    const int wlo = max(0, r0 - AW_HALO), whi = min(n, r0 + AW_ROWS + AW_HALO);
    for (int t = threadIdx.x; t < whi - wlo; t += 256) win[t] = Y[wlo + t];
    __syncthreads();
    const int sub = (int)(threadIdx.x % AW_LPR);
    constexpr int GROUPS = 256 / AW_LPR;
    // every 16-lane group works on AW_DUAL rows at a time so that twice as many loads are in flight
    for (int rr = (int)threadIdx.x / AW_LPR; rr < AW_ROWS; rr += GROUPS * AW_DUAL) {
        int row[AW_DUAL], j0[AW_DUAL], e[AW_DUAL];
        float2 yi[AW_DUAL];
        float ax[AW_DUAL], ay[AW_DUAL];
        bool more = false;
#pragma unroll
        for (int d = 0; d < AW_DUAL; ++d) {
            row[d] = r0 + rr + d * GROUPS;
            const bool live = rr + d * GROUPS < AW_ROWS && row[d] < n;
            if (!live) row[d] = -1;
            j0[d] = live ? row_ptr[row[d]] + sub : 0;
            e[d] = live ? row_ptr[row[d] + 1] : 0;
            yi[d] = live ? win[row[d] - wlo] : make_float2(0.f, 0.f);
            ax[d] = ay[d] = 0.f;
            more |= j0[d] < e[d];
        }
        while (__any(more)) {
            int c[AW_DUAL][AW_U];
            float v[AW_DUAL][AW_U];
            float2 yj[AW_DUAL][AW_U];
#pragma unroll
            for (int d = 0; d < AW_DUAL; ++d)
#pragma unroll
                for (int q = 0; q < AW_U; ++q) {
                    const int j = j0[d] + q * AW_LPR;
                    const bool in = j < e[d];
                    c[d][q] = in ? col[j] : wlo;      // padding: any in-window point, weight 0
                    v[d][q] = in ? val[j] : 0.f;
                }
#pragma unroll
            for (int d = 0; d < AW_DUAL; ++d)
#pragma unroll
                for (int q = 0; q < AW_U; ++q) {
                    const unsigned off = (unsigned)(c[d][q] - wlo);
                    if (off < (unsigned)(whi - wlo)) yj[d][q] = win[off];
                    else yj[d][q] = Y[min((uint32_t)c[d][q], (uint32_t)n - 1u)];
                }
            more = false;
#pragma unroll
            for (int d = 0; d < AW_DUAL; ++d) {
#pragma unroll
                for (int q = 0; q < AW_U; ++q) {
                    const float dx = yi[d].x - yj[d][q].x, dy = yi[d].y - yj[d][q].y;
                    const float w = __builtin_amdgcn_rcpf(fmaf(dy, dy, fmaf(dx, dx, 1.0f)));
                    const float pw = v[d][q] * w;
                    ax[d] = fmaf(pw, dx, ax[d]);
                    ay[d] = fmaf(pw, dy, ay[d]);
                }
                j0[d] += AW_LPR * AW_U;
                more |= j0[d] < e[d];
            }
        }
#pragma unroll
        for (int d = 0; d < AW_DUAL; ++d) {
#pragma unroll
            for (int o = AW_LPR / 2; o > 0; o >>= 1) {
                ax[d] += __shfl_xor(ax[d], o, WAVE);
                ay[d] += __shfl_xor(ay[d], o, WAVE);
            }
            if (row[d] >= 0 && sub == 0) A[row[d]] = make_float2(ax[d], ay[d]);
        }
    }
}

hipError_t launch_attract(tsne_ctx *c, const float *d_Y, hipStream_t s)
{
    const int n = c->p.n;
    (void)d_Y;
    if (c->reorder_on && !c->identity) {
        hipLaunchKernelGGL(attract_csr_window, dim3((n + AW_ROWS - 1) / AW_ROWS), dim3(256), 0, s, c->row_ptr, c->col,
                           c->val, c->Yi, n, c->A);
    } else {
        const unsigned blocks = (unsigned)(((int64_t)n * AW_LPR + 255) / 256);
        hipLaunchKernelGGL((attract_csr<AW_LPR, AW_U>), dim3(blocks), dim3(256), 0, s, c->row_ptr, c->col, c->val,
                           c->Yi, n, c->row_order, c->A);
    }
    return hipGetLastError();
}

// Alg. 1 line 8.  grad = 4 (alpha A - R / Z) (Eq. (7)); per coordinate the gain grows by
// gain_inc when gradient and velocity differ in sign (sign in {-1,0,+1}) and is multiplied by
// gain_dec otherwise, floored at gain_min; velocity = momentum velocity - lr gain grad;
// y += velocity.
__device__ __forceinline__ int sign3(float v) { return v > 0.f ? 1 : (v < 0.f ? -1 : 0); }

__global__ __launch_bounds__(256) void update_k(float2 *__restrict__ Y, const uint32_t *__restrict__ orig,
                                                const float2 *__restrict__ Yi, float2 *__restrict__ uY,
                                                float2 *__restrict__ gains, const float2 *__restrict__ A,
                                                const float2 *__restrict__ R, const double *__restrict__ Z, int n,
                                                float alpha, float momentum, float lr, float gain_inc, float gain_dec,
                                                float gain_min)
{
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n) return;
    const float invZ = (float)(1.0 / *Z);
    const float2 a = A[s], r = R[s];
    float2 g = gains[s], u = uY[s], y = Yi[s];
    const float gx = 4.0f * (alpha * a.x - r.x * invZ), gy = 4.0f * (alpha * a.y - r.y * invZ);
    g.x = (sign3(gx) != sign3(u.x)) ? g.x + gain_inc : g.x * gain_dec;
    g.y = (sign3(gy) != sign3(u.y)) ? g.y + gain_inc : g.y * gain_dec;
    g.x = fmaxf(g.x, gain_min); g.y = fmaxf(g.y, gain_min);
    u.x = momentum * u.x - lr * g.x * gx;
    u.y = momentum * u.y - lr * g.y * gy;
    gains[s] = g;
    uY[s] = u;
    y.x += u.x; y.y += u.y;
    Y[min(orig[s], (uint32_t)n - 1u)] = y;
}

hipError_t launch_update(tsne_ctx *c, float *d_Y, float alpha, float momentum, hipStream_t s)
{
    const int n = c->p.n;
    hipLaunchKernelGGL(update_k, dim3((n + 255) / 256), dim3(256), 0, s, (float2 *)d_Y, c->orig[c->cur_state], c->Yi,
                       c->uYb[c->cur_state], c->gainsb[c->cur_state], c->A, c->R, c->Z, n, alpha, momentum, c->p.lr,
                       c->p.gain_inc, c->p.gain_dec, c->p.gain_min);
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
