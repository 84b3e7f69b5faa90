// Sec. III-C step 5 of the paper on gfx950: repulsive forces and the Z estimate by a
// Barnes-Hut walk, one wavefront per group of 64 consecutive points of the spatial order.
//
// A cell is accepted for a group when Eq. (14) (side^2 < theta^2 |y_i - y_cell|^2, y_cell the
// centre of mass) holds for every point of the group, so all 64 lanes always take the same
// path.  The walk alternates between two roles so that no lane ever waits on a pointer chase:
//
//   lanes = cells    up to 64 cells are popped from the wave's stack and tested at once.
//        sift        two cheap tests.  Against the group's bounding box: the distance from y_cell
//                    to the box is a lower bound of the distance to every point, and every step
//                    of the single-precision test is monotone, so passing here implies passing
//                    for each point, bit for bit.  Against four witness points of the group: if
//                    one of them fails Eq. (14) the cell is rejected.  The few cells neither
//                    test decides wait on a short pending list.
//        settle      64 pending cells at a time: minimum of |y_i - y_cell|^2 over the group's
//                    points (LDS broadcasts), then the exact test.
//                    Either way accepted cells go to a list in LDS as (y_cell, N_cell);
//                    rejected inner cells push their children; rejected leaves put their
//                    points on a second list.
//   lanes = points   the lists are drained: every lane adds N w^2 (y_i - y_cell) and N w,
//                    w = 1/(1+|y_i - y_cell|^2), for its own point (Eq. (15) and the Z note
//                    that follows it); list entries are LDS broadcasts.
//
// The LDS arrays of a wave are sized to seven allocation granules (1280 bytes each) and the
// kernel is held to 96 registers: with those numbers 14 walking waves fit on a compute unit
// beside one workgroup of the attraction kernel, and 18 alone.
//
// A point meets itself exactly once (the leaf that holds it can never pass its own test when
// theta^2 < 1/2) with w = 1 and zero force; the Z accumulator therefore starts at -1.
#include "tsne_internal.h"

#include <math.h>

constexpr int WALK_STACK = 512;      // stack entries
constexpr int WALK_SLACK = 3 * MAX_GRID_BITS;   // head room for a depth-first descent (3 entries per level)
constexpr int WALK_PEND = 128;       // pending list entries
constexpr int WALK_FAST_LEAF = 8;    // leaves up to this size are copied by their own lane
constexpr int WALK_CLIST = 96;       // accepted cells waiting for the drain (16 B each), >= 64
constexpr int WALK_PLIST = 512;      // points of opened leaves waiting (8 B each), >= 64 * WALK_FAST_LEAF
static_assert(WALK_CLIST >= WAVE && WALK_PLIST >= WAVE * WALK_FAST_LEAF, "one round must fit");
static_assert(WAVE * WALK_FAST_LEAF < 65536, "two counts share one prefix sum");

// side^2 < theta^2 * d2, with d2 = fma(dy, dy, dx*dx): one rounding per operation.
__device__ __forceinline__ float dist2_rounded(float dx, float dy)
{
#pragma clang fp contract(off)
    float dx2 = dx * dx;
    return fmaf(dy, dy, dx2);
}

__device__ __forceinline__ bool passes(float side2, float theta2, float d2)
{
#pragma clang fp contract(off)
    float rhs = theta2 * d2;
    return side2 < rhs;
}

// One interaction: y_cell (c.x, c.y) with weight c.z = N_cell.
#define TSNE_INTERACT(c)                                                      \
    {                                                                         \
        const float dx_ = x - (c).x, dy_ = y - (c).y;                         \
        const float q_ = __builtin_amdgcn_rcpf(fmaf(dy_, dy_, fmaf(dx_, dx_, 1.0f))); \
        z = fmaf((c).z, q_, z);                                               \
        const float f_ = (c).z * q_ * q_;                                     \
        fx = fmaf(f_, dx_, fx);                                               \
        fy = fmaf(f_, dy_, fy);                                               \
    }

// The same for a single point (weight 1).
#define TSNE_INTERACT1(c)                                                     \
    {                                                                         \
        const float dx_ = x - (c).x, dy_ = y - (c).y;                         \
        const float q_ = __builtin_amdgcn_rcpf(fmaf(dy_, dy_, fmaf(dx_, dx_, 1.0f))); \
        z += q_;                                                              \
        const float f_ = q_ * q_;                                             \
        fx = fmaf(f_, dx_, fx);                                               \
        fy = fmaf(f_, dy_, fy);                                               \
    }

// lanes = points: every lane adds the listed cells' (points') contributions for its own point.
// Two register sets take turns: one is filled from LDS while the other is used.
__device__ __forceinline__ void drain_cells(const float4 *__restrict__ list, int cnt, float x, float y, float &fx,
                                            float &fy, float &z)
{
    __syncthreads();
    int e = 0;
    if (cnt >= 8) {
        float4 a0 = list[0], a1 = list[1], a2 = list[2], a3 = list[3];
        for (e = 4; e + 8 <= cnt; e += 8) {
            const float4 b0 = list[e], b1 = list[e + 1], b2 = list[e + 2], b3 = list[e + 3];
            TSNE_INTERACT(a0) TSNE_INTERACT(a1) TSNE_INTERACT(a2) TSNE_INTERACT(a3)
            a0 = list[e + 4]; a1 = list[e + 5]; a2 = list[e + 6]; a3 = list[e + 7];
            TSNE_INTERACT(b0) TSNE_INTERACT(b1) TSNE_INTERACT(b2) TSNE_INTERACT(b3)
        }
        TSNE_INTERACT(a0) TSNE_INTERACT(a1) TSNE_INTERACT(a2) TSNE_INTERACT(a3)
    }
    for (; e < cnt; ++e) {
        const float4 c = list[e];
        TSNE_INTERACT(c)
    }
    __syncthreads();
}

__device__ __forceinline__ void drain_points(const float2 *__restrict__ list, int cnt, float x, float y, float &fx,
                                             float &fy, float &z)
{
    __syncthreads();
    int e = 0;
    if (cnt >= 8) {
        float2 a0 = list[0], a1 = list[1], a2 = list[2], a3 = list[3];
        for (e = 4; e + 8 <= cnt; e += 8) {
            const float2 b0 = list[e], b1 = list[e + 1], b2 = list[e + 2], b3 = list[e + 3];
            TSNE_INTERACT1(a0) TSNE_INTERACT1(a1) TSNE_INTERACT1(a2) TSNE_INTERACT1(a3)
            a0 = list[e + 4]; a1 = list[e + 5]; a2 = list[e + 6]; a3 = list[e + 7];
            TSNE_INTERACT1(b0) TSNE_INTERACT1(b1) TSNE_INTERACT1(b2) TSNE_INTERACT1(b3)
        }
        TSNE_INTERACT1(a0) TSNE_INTERACT1(a1) TSNE_INTERACT1(a2) TSNE_INTERACT1(a3)
    }
    for (; e < cnt; ++e) {
        const float2 c = list[e];
        TSNE_INTERACT1(c)
    }
    __syncthreads();
}

// The walk of one group g.  stack / pend / pts / clist / plist are the wave's LDS arrays.
__device__ __forceinline__ void walk_group(const int g, uint32_t *stack, uint32_t *pend, float2 *pts, float4 *clist,
                                           float2 *plist,
                                           const Cell *__restrict__ cells, const float2 *__restrict__ Ys,
                                           const uint32_t *__restrict__ perm, int n, const float4 *__restrict__ root,
                                           float theta2, const uint32_t *__restrict__ ncells, uint32_t cap_cells,
                                           float2 *__restrict__ R, double *__restrict__ zpart, uint32_t *status)
{
    const int lane = (int)threadIdx.x;
    const int p = g * WAVE + lane;
    const bool valid = p < n;
    const uint32_t m_cells = *ncells;
    if (m_cells > cap_cells || m_cells == 0u) {   // tree did not fit: flagged by the build, produce zeros
        if (valid) R[min(perm[p], (uint32_t)n - 1u)] = make_float2(0.f, 0.f);
        if (lane == 0) zpart[g] = 0.0;
        return;
    }
    __syncthreads();   // the previous group of this wave is done with the LDS arrays
    // own point; idle lanes of the last group shadow its first point and are never written out
    const float2 me = Ys[valid ? p : g * WAVE];
    const float x = me.x, y = me.y;
    pts[lane] = me;
    const float bx0 = wave_min(x), bx1 = wave_max(x), by0 = wave_min(y), by1 = wave_max(y);
    const float W = root->z;
    // z: the terms of one batch in single precision, moved to the double zsum after every batch (a point's sum over
    // tens of thousands of nearly equal terms -- theta = 0, or Y0 where every q is close to 1 -- otherwise picks up
    // the same rounding error at every addition: 1e-4 of Z at 20,000 points).  Starts at -1: the point meets itself
    // among the members of its own leaf.
    float fx = 0.f, fy = 0.f, z = 0.f;
    double zsum = -1.0;
    int sp = 1, np = 0, icc = 0, icp = 0;   // wave-uniform; kept in scalar registers via readfirstlane
    bool overflow = false;
    uint32_t rounds = 0;
    if (lane == 0) stack[0] = 0u;
    __syncthreads();
    // four members of the group used as quick witnesses: if Eq. (14) fails for one of them the
    // cell is rejected for the group without looking at the other 60
    const float2 w0 = pts[0], w1 = pts[21], w2 = pts[42], w3 = pts[63];
    while (sp > 0 || np > 0) {
        // every cell is popped from the stack at most once and from the pending list at most
        // once, so more rounds than 2 * cells means a malformed tree; ids and member positions
        // are clamped so that even then no access leaves the arrays
        if (++rounds > 2u * m_cells + 2u) { overflow = true; break; }
        // Stack bound: every popped cell pushes at most 4 children.  A round takes as many
        // cells as still leave WALK_SLACK entries free afterwards whatever they push; when not
        // even one cell fits that rule the wave takes the single top cell per round -- plain
        // depth-first search, which adds at most 3 entries per level below the popped cell
        // (<= 69 for 24 levels) before it shrinks again.  So sp never passes WALK_STACK - 3.
        const int room = WALK_STACK - WALK_SLACK - sp;
        const bool pressure = room < 3;
        const bool from_pending = room >= 4 && (np >= WAVE || sp == 0);
        // (np >= 64 in a stack round only happens when the stack is nearly full: settle at once,
        //  so that the pending list cannot outgrow its 128 entries)
        const bool exact = from_pending || pressure || np >= WAVE;
        int take;
        uint32_t id;
        if (from_pending) {
            take = min(min(np, WAVE), room >> 2);            // pending cells free no stack entry
            id = lane < take ? pend[np - take + lane] : 0u;
            np -= take;
        } else {
            take = pressure ? 1 : min(min(sp, WAVE), room / 3);   // a popped cell nets at most +3
            id = lane < take ? stack[sp - take + lane] : 0u;
            sp -= take;
        }
        const bool act = lane < take;
        id = min(id, m_cells - 1u);
        const uint4 *cp = reinterpret_cast<const uint4 *>(cells + id);
        const uint4 ca = cp[0], cb = cp[1];
        const float cx = __uint_as_float(ca.x), cy = __uint_as_float(ca.y);
        const uint32_t cnt = ca.z;
        const bool leaf = (ca.w >> 8) & 1u;
        const float side = ldexpf(W, -(int)(ca.w & 0xFFu));   // exact: W is a power of two
        const float side2 = side * side;
        bool pass, decided;
        if (exact) {
            // settle: minimum squared distance from y_cell to the 64 points of the group
            float dmin = INFINITY;
#pragma unroll 8
            for (int i = 0; i < WAVE; ++i) {
                const float2 q = pts[i];
                dmin = fminf(dmin, dist2_rounded(q.x - cx, q.y - cy));
            }
            pass = passes(side2, theta2, dmin);
            decided = true;
        } else {
            // sift: the bounding box settles most acceptances, the witnesses most rejections
            const float dx = fmaxf(fmaxf(bx0 - cx, cx - bx1), 0.0f);
            const float dy = fmaxf(fmaxf(by0 - cy, cy - by1), 0.0f);
            pass = passes(side2, theta2, dist2_rounded(dx, dy));
            const float dw = fminf(fminf(dist2_rounded(w0.x - cx, w0.y - cy), dist2_rounded(w1.x - cx, w1.y - cy)),
                                   fminf(dist2_rounded(w2.x - cx, w2.y - cy), dist2_rounded(w3.x - cx, w3.y - cy)));
            decided = pass || !passes(side2, theta2, dw);
        }
        const bool acc = act && pass;
        const bool und = act && !decided;
        const bool open = act && decided && !pass && leaf;
        const bool desc = act && decided && !pass && !leaf;
        const bool ofast = open && cnt <= (uint32_t)WALK_FAST_LEAF;
        const uint64_t macc = __ballot(acc);
        // one prefix sum for two lists: members of small opened leaves (low half: at most 64 * WALK_FAST_LEAF) and
        // children of rejected inner cells (high half: at most 256)
        const int nch = desc ? 1 + (cb.y != TSNE_NONE) + (cb.z != TSNE_NONE) + (cb.w != TSNE_NONE) : 0;
        int both_tot;
        const int both_off = wave_excl_scan((ofast ? (int)cnt : 0) | (nch << 16), &both_tot);
        both_tot = __builtin_amdgcn_readfirstlane(both_tot);
        const int moff = both_off & 0xFFFF, mtot = both_tot & 0xFFFF;
        const int nacc = __popcll(macc);
        if (icc + nacc > WALK_CLIST) { drain_cells(clist, icc, x, y, fx, fy, z); icc = 0; zsum += (double)z; z = 0.f; }
        if (acc) clist[icc + __popcll(macc & lanemask_lt())] = make_float4(cx, cy, (float)cnt, 0.f);
        icc = __builtin_amdgcn_readfirstlane(icc + nacc);
        if (icp + mtot > WALK_PLIST) { drain_points(plist, icp, x, y, fx, fy, z); icp = 0; zsum += (double)z; z = 0.f; }
        if (ofast) {
            float2 q[WALK_FAST_LEAF];
#pragma unroll
            for (int j = 0; j < WALK_FAST_LEAF; ++j)
                q[j] = Ys[min(cb.x + (uint32_t)j, (uint32_t)n - 1u)];
#pragma unroll
            for (int j = 0; j < WALK_FAST_LEAF; ++j)
                if ((uint32_t)j < cnt) plist[icp + moff + j] = q[j];
        }
        icp = __builtin_amdgcn_readfirstlane(icp + mtot);
        // undecided cells wait for a full batch (only met in sift rounds, where np < 64)
        const uint64_t mund = __ballot(und);
        if (und) pend[np + __popcll(mund & lanemask_lt())] = id;
        np = __builtin_amdgcn_readfirstlane(np + __popcll(mund));
        // Large leaves (only at the maximum depth, or when leaf_cap > WALK_FAST_LEAF).  Their members
        // are consecutive positions; the lanes copy the concatenation of all of them, 64 points a
        // step: a prefix sum gives every leaf its offset, and lane t finds its leaf as the last
        // lane whose offset is <= t (other lanes have empty segments, which the search skips).
        const bool big = open && !ofast;
        if (__any(big)) {
            int tbig;
            // (leaves of one round are different cells, so their sizes add up to at most n)
            const int boff = wave_excl_scan(big ? (int)cnt : 0, &tbig);
            tbig = __builtin_amdgcn_readfirstlane(tbig);
            for (int base = 0; base < tbig;) {
                if (WALK_PLIST - icp < WAVE) { drain_points(plist, icp, x, y, fx, fy, z); icp = 0; zsum += (double)z; z = 0.f; }
                const int take = min(tbig - base, WALK_PLIST - icp);
                for (int k = 0; k < take; k += WAVE) {
                    const int t = base + k + lane;
                    const int tt = min(t, tbig - 1);
                    int owner = 0;
#pragma unroll
                    for (int s = WAVE / 2; s > 0; s >>= 1) {
                        const int c = owner + s;            // < 64: owner + s never passes 63
                        if (__shfl(boff, c, WAVE) <= tt) owner = c;
                    }
                    const uint32_t first = __shfl(cb.x, owner, WAVE);
                    const int ooff = __shfl(boff, owner, WAVE);
                    if (t < base + take)
                        plist[icp + k + lane] = Ys[min(first + (uint32_t)(tt - ooff), (uint32_t)n - 1u)];
                }
                icp = __builtin_amdgcn_readfirstlane(icp + take);
                base += take;
            }
        }
        // children of rejected inner cells
        const int coff = both_off >> 16, ctot = both_tot >> 16;
        if (sp + ctot > WALK_STACK) { overflow = true; break; }   // unreachable for a well-formed tree
        if (desc) {
            int o = sp + coff;
            stack[o++] = id + 1u;
            if (cb.y != TSNE_NONE) stack[o++] = cb.y;
            if (cb.z != TSNE_NONE) stack[o++] = cb.z;
            if (cb.w != TSNE_NONE) stack[o++] = cb.w;
        }
        sp = __builtin_amdgcn_readfirstlane(sp + ctot);
        __syncthreads();
    }
    if (overflow) {
        if (lane == 0) atomicOr(status, TSNE_STATUS_WALK_OVERFLOW);
        fx = fy = 0.f; z = 0.f; zsum = 0.0; icc = icp = 0;
    }
    drain_cells(clist, icc, x, y, fx, fy, z);
    zsum += (double)z; z = 0.f;
    drain_points(plist, icp, x, y, fx, fy, z);
    zsum += (double)z;
    if (valid) R[min(perm[p], (uint32_t)n - 1u)] = make_float2(fx, fy);
    double zd = wave_sum(valid ? zsum : 0.0);
    if (lane == 0) zpart[g] = zd;
}

// One wave per workgroup.  With a work counter the grid is a fixed number of resident waves that
// take groups from the counter until none is left (every wave ends when the counter has passed
// the number of groups); without one, workgroup g walks group g.
__global__ __attribute__((amdgpu_waves_per_eu(5))) __launch_bounds__(WAVE) void bh_walk(const Cell *__restrict__ cells, const float2 *__restrict__ Ys,
                                                const uint32_t *__restrict__ perm, int n,
                                                const float4 *__restrict__ root, float theta2,
                                                const uint32_t *__restrict__ ncells, uint32_t cap_cells,
                                                float2 *__restrict__ R, double *__restrict__ zpart,
                                                uint32_t *status, uint32_t *counter)
{
    __shared__ uint32_t stack[WALK_STACK];
    __shared__ uint32_t pend[WALK_PEND];
    __shared__ float2 pts[WAVE];
    __shared__ float4 clist[WALK_CLIST];
    __shared__ float2 plist[WALK_PLIST];
    const int ngroups = (n + WAVE - 1) / WAVE;
    if (!counter) {
        walk_group((int)blockIdx.x, stack, pend, pts, clist, plist, cells, Ys, perm, n, root, theta2, ncells, cap_cells, R,
                   zpart, status);
        return;
    }
    // The first group of a wave is its workgroup number; further groups come from counters.
    // (All waves start together: if each began with a draw, thousands of atomics on one address
    // would queue up and the last wave would start tens of microseconds late.)  Same-address
    // atomics are served one after the other, about one every 20 ns, which 20 000 draws in a
    // third of a millisecond would saturate: the groups are dealt into WALK_COUNTERS classes
    // (group mod WALK_COUNTERS), each with its own counter and its own share of the waves.
    // The grid is a multiple of WALK_COUNTERS, so every class has grid / WALK_COUNTERS waves.
    __shared__ uint32_t next_group;
    const uint32_t cls = blockIdx.x % WALK_COUNTERS, dealt = gridDim.x / WALK_COUNTERS;
    uint32_t g = blockIdx.x;
    while (g < (uint32_t)ngroups) {
        walk_group((int)g, stack, pend, pts, clist, plist, cells, Ys, perm, n, root, theta2, ncells, cap_cells, R, zpart,
                   status);
        // lane 0 draws the next group of the class; every lane reads the number back from LDS
        __syncthreads();
        if (threadIdx.x == 0) next_group = cls + WALK_COUNTERS * (dealt + atomicAdd(counter + cls, 1u));
        __syncthreads();
        g = (uint32_t)__builtin_amdgcn_readfirstlane((int)next_group);
    }
}

// Z = sum of the per-group partial sums, in a fixed order (thread t takes groups t, t + 1024, ...,
// eight running sums so that eight loads are in flight, combined pairwise).
__global__ __launch_bounds__(1024) void z_final(const double *__restrict__ zpart, int ngroups, double *__restrict__ Z)
{
    __shared__ double ws[16];
    double acc[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    for (int i = (int)threadIdx.x; i < ngroups; i += 8 * 1024) {
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] += i + 1024 * k < ngroups ? zpart[i + 1024 * k] : 0.0;
    }
    double a = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
    a = wave_sum(a);
    if (lane_id() == 0) ws[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int k = 0; k < 16; ++k) t += ws[k];
        *Z = t;
    }
}

hipError_t launch_walk(tsne_ctx *c, hipStream_t s)
{
    const int n = c->p.n;
    const int ngroups = (n + WAVE - 1) / WAVE;
    const float theta2 = c->p.theta * c->p.theta;
    // walk_resident > 0: that many resident waves per compute unit share the groups through a
    // counter (zeroed by the tree build), which leaves a known part of every unit to the attraction
    const bool resident = c->p.walk_resident > 0 && ngroups > c->p.walk_resident * c->num_cu &&
                          c->p.walk_resident * c->num_cu >= WALK_COUNTERS;
    const int grid = resident ? c->p.walk_resident * c->num_cu / WALK_COUNTERS * WALK_COUNTERS : ngroups;
    hipLaunchKernelGGL(bh_walk, dim3(grid), dim3(WAVE), 0, s, c->cells, c->Ys, c->perm, n, c->root,
                       theta2, c->ncells, (uint32_t)c->cap_cells, c->R, c->zpart, c->status,
                       resident ? c->walk_counter : (uint32_t *)nullptr);
    hipLaunchKernelGGL(z_final, dim3(1), dim3(1024), 0, s, c->zpart, ngroups, c->Z);
    return hipGetLastError();
}
