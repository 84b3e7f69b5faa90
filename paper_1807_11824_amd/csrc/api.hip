// C ABI of the library (include/tsne.h): argument checks, workspace carve-up and the
// order in which the kernels of one iteration are enqueued (Alg. 1 lines 3-9).
#include "tsne_internal.h"

#include <algorithm>

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

namespace {

constexpr size_t ALIGN = 256;
constexpr int KL_PART_DOUBLES = 3 * 1024;

size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

// Most cells a tree over n points can have: its leaves are disjoint and non-empty (at most n), and an
// inner cell holds more than leaf_cap points, so each of the `bits` levels above the deepest has at
// most n / (leaf_cap + 1) of them.
int64_t cell_capacity(int64_t n, int bits, int64_t leaf_cap)
{
    return n + (int64_t)bits * (n / (leaf_cap + 1)) + 1;
}

// Walks the workspace layout; with base == nullptr it only measures.
size_t carve(tsne_ctx *c, const tsne_params *p, char *base)
{
    const size_t n = (size_t)p->n;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *ptr = base ? base + off : nullptr;
        off += up(bytes);
        return (void *)ptr;
    };
    const int32_t cap = (int32_t)cell_capacity(p->n, p->morton_bits, p->leaf_cap);   // < 2^31: check_params
    const size_t nblk_sort = (n + SORT_TILE_MIN - 1) / SORT_TILE_MIN;   // the most tiles any tile size gives
    const size_t nblk_lev = (n + LEVEL_TILE - 1) / LEVEL_TILE;
    const size_t ngroups = (n + WAVE - 1) / WAVE;
    void *q;
    const size_t nbox = std::max<size_t>(BBOX_MAX_BLOCKS, (n + 255) / 256);
    q = take(sizeof(float4) * 2 * nbox);             if (c) c->bbox_part = (float4 *)q;
    q = take(sizeof(float4));                        if (c) c->root = (float4 *)q;
    q = take(sizeof(uint32_t));                      if (c) c->status = (uint32_t *)q;
    q = take(sizeof(uint32_t));                      if (c) c->ncells = (uint32_t *)q;
    for (int k = 0; k < 2; ++k) { q = take(8 * n); if (c) c->words[k] = (uint64_t *)q; }
    q = take(4 * n);                                 if (c) c->perm = (uint32_t *)q;
    q = take(4 * n);                                 if (c) c->row_order = (uint32_t *)q;
    q = take(4 * (size_t)RADIX * nblk_sort);         if (c) c->hist = (uint32_t *)q;
    q = take(4 * (size_t)RADIX);                     if (c) c->dtot = (uint32_t *)q;
    q = take(8 * n);                                 if (c) c->Ys = (float2 *)q;
    q = take(2 * n);                                 if (c) c->lev = (uint16_t *)q;
    q = take(sizeof(ScanPart) * nblk_lev);           if (c) c->part = (ScanPart *)q;
    q = take(4 * (n + 1));                           if (c) c->cellseq = (uint32_t *)q;
    q = take(16 * (n + 1));                          if (c) c->ps = (double2 *)q;
    q = take(sizeof(Cell) * (size_t)cap);            if (c) { c->cells = (Cell *)q; c->cap_cells = cap; }
    q = take(4 * (size_t)cap);                       if (c) c->cell_p = (uint32_t *)q;
    q = take((size_t)cap);                           if (c) c->cell_t = (uint8_t *)q;
    const int32_t big_cap = (int32_t)(n / 8 + 1024);
    q = take((1 + WALK_COUNTERS) * sizeof(uint32_t));                  if (c) { c->big_count = (uint32_t *)q; c->walk_counter = c->big_count + 1; }
    q = take(sizeof(uint2) * (size_t)big_cap);       if (c) { c->big_list = (uint2 *)q; c->big_cap = big_cap; }
    q = take(8 * n);                                 if (c) c->R = (float2 *)q;
    q = take(8 * n);                                 if (c) c->A = (float2 *)q;
    q = take(8 * n);                                 if (c) c->Yi = (float2 *)q;
    const bool reorder = (p->reorder_every > 0 || p->graph_order_iters > 0) && p->max_nnz > 0;
    for (int k = 0; k < (reorder ? 2 : 1); ++k) {
        q = take(8 * n); if (c) c->uYb[k] = (float2 *)q;
        q = take(8 * n); if (c) c->gainsb[k] = (float2 *)q;
        q = take(4 * n); if (c) c->orig[k] = (uint32_t *)q;
    }
    if (reorder) {
        const size_t m = (size_t)p->max_nnz;
        const size_t ms = m + (ATTRACT_CHUNK - 1) * n + ATTRACT_SLACK;   // near rows are padded to whole chunks
        q = take(4 * n); if (c) c->inv = (uint32_t *)q;
        q = take(4 * n); if (c) c->len_near = (int32_t *)q;
        q = take(4 * n); if (c) c->len_far = (int32_t *)q;
        q = take(4 * (n + 1)); if (c) c->rp_near = (int32_t *)q;
        q = take(4 * (n + 1)); if (c) c->rp_far = (int32_t *)q;
        q = take(4 * n);       if (c) c->far_rows = (uint32_t *)q;
        q = take(4);           if (c) c->far_count = (uint32_t *)q;
        q = take(8 * n);       if (c) c->Afar = (float2 *)q;
        q = take(2 * ms);      if (c) c->col_near = (uint16_t *)q;
        q = take(4 * (m + ATTRACT_SLACK)); if (c) c->col_far = (int32_t *)q;
        q = take(4 * ms);      if (c) c->val_s = (float *)q;
        if (c) c->ft_tiles = 0;
        if (ft_possible(p)) {
            const size_t nrt = (n + FT_ROWS - 1) / FT_ROWS, nct = (n + FT_COLS - 1) / FT_COLS;
            if (c) { c->ft_tiles = (int64_t)(nrt * nct); c->ft_nct = (int)nct; }
            q = take(4 * nrt * nct);       if (c) c->ft_cnt = (uint32_t *)q;
            q = take(4 * (nrt * nct + 1)); if (c) c->ft_ptr = (int32_t *)q;
            q = take(4 * m);               if (c) c->ft_col = (int32_t *)q;
            q = take(2 * m);               if (c) c->ft_row = (uint16_t *)q;
            q = take(4 * m);               if (c) c->ft_val = (float *)q;
            q = take(16 * n);              if (c) c->ft_acc = (double *)q;
            q = take(32);                  if (c) c->ft_meta = (uint32_t *)q;
        }
    }
    q = take(4 * (ATTRACT_MAX_PARTS + 1));           if (c) c->arow = (int32_t *)q;
    q = take(8 * ngroups);                           if (c) c->zpart = (double *)q;
    q = take(8);                                     if (c) c->Z = (double *)q;
    q = take(8 * KL_PART_DOUBLES);                   if (c) c->kl_part = (double *)q;
    return off;
}

// bits needed for the numbers 0 .. n-1
int index_bits(int64_t n)
{
    int b = 0;
    while (((int64_t)1 << b) < n) ++b;
    return b;
}

int check_params(const tsne_params *p)
{
    if (!p) return TSNE_EINVAL;
    // (several kernels run 16 lanes per point in one launch, and a launch axis holds fewer than 2^32 work-items)
    if (p->n < 1 || p->n > (1 << 27)) return TSNE_EINVAL;
    if (!(p->theta >= 0.0f) || p->theta > 0.7f) return TSNE_EINVAL;
    if (p->morton_bits < 1 || p->morton_bits > MAX_GRID_BITS) return TSNE_EINVAL;
    // a point's grid key and its number share one 64-bit word in the sort
    if (2 * p->morton_bits + index_bits(p->n) > 64) return TSNE_EINVAL;
    if (p->leaf_cap < 1) return TSNE_EINVAL;
    if (p->overlap < 0 || p->overlap > 1) return TSNE_EINVAL;
    if (cell_capacity(p->n, p->morton_bits, p->leaf_cap) > 0x7FFFFFFFll) return TSNE_EINVAL;   // cells are numbered in 32 bits
    if (p->reorder_every < 0 || p->graph_order_iters < 0 || p->graph_order_iters > 1000) return TSNE_EINVAL;
    if (p->attract_resident < 0 || p->attract_resident > 64) return TSNE_EINVAL;
    if (p->walk_resident < 0 || p->walk_resident > 32) return TSNE_EINVAL;
    if (p->far_tiles < 0 || p->far_tiles > 2) return TSNE_EINVAL;
    if (p->max_nnz < 0 || p->max_nnz > 0x7FFFFFFFll) return TSNE_EINVAL;
    // the renumbered copy pads every row to whole chunks and is indexed with int32
    if (p->max_nnz > 0 && p->max_nnz + (ATTRACT_CHUNK - 1ll) * p->n + ATTRACT_SLACK > 0x7FFFFFFFll) return TSNE_EINVAL;
    if (!isfinite(p->lr) || !isfinite(p->exaggeration) || !isfinite(p->momentum_early) ||
        !isfinite(p->momentum_late) || !isfinite(p->gain_inc) || !isfinite(p->gain_dec) || !isfinite(p->gain_min))
        return TSNE_EINVAL;
    return TSNE_OK;
}

int fail_hip(tsne_ctx *c, hipError_t e, const char *where)
{
    if (c) snprintf(c->err, sizeof(c->err), "%s: %s", where, hipGetErrorString(e));
    return TSNE_EHIP;
}

int fail(tsne_ctx *c, int code, const char *msg)
{
    if (c) snprintf(c->err, sizeof(c->err), "%s", msg);
    return code;
}

// Events of one timed step: 0 start, 1 tree built, 2 walk done, 3 / 4 streaming part of the attraction,
// 5 update done, 6 / 7 far part of the attraction, 8 update started.
constexpr int NEV = 9;

// Forces at d_Y into c->A, c->R, c->Z.  The attraction only needs Y and P, so with overlap it runs
// on the second stream: the small far part beside the tree build (the tree kernels are short and
// latency-bound; a few gathering workgroups do not slow them much) and the streaming part beside
// the walk, whose arithmetic and the attraction's memory traffic use different parts of the chip.
int enqueue_forces(tsne_ctx *c, const float *d_Y, hipEvent_t *ev, bool cached = false)
{
    hipError_t e;
    const bool two = c->p.overlap && c->stream2;
    hipStream_t sa = two ? c->stream2 : c->stream;   // where the attraction runs
    auto fork = [&](hipEvent_t evt) -> int {
        if ((e = hipEventRecord(evt, c->stream)) != hipSuccess) return fail_hip(c, e, "event record");
        if ((e = hipStreamWaitEvent(c->stream2, evt, 0)) != hipSuccess) return fail_hip(c, e, "stream wait");
        return TSNE_OK;
    };
    // The bucketed far part needs nothing but Y and the root square: with two streams it starts beside the tree build
    // (which hides behind it), not behind the walk.
    const bool tiles_early = two && c->ft_active && c->p.n > SMALL_SORT_MAX;
    auto farpart = [&]() -> int {
        if (ev) (void)hipEventRecord(ev[6], sa);
        if ((e = launch_attract_far(c, sa, tiles_early)) != hipSuccess) return fail_hip(c, e, "attract (far part)");
        if (ev) (void)hipEventRecord(ev[7], sa);
        return TSNE_OK;
    };
    auto mainpart = [&]() -> int {
        if (ev) (void)hipEventRecord(ev[3], sa);
        if ((e = launch_attract_main(c, sa, !tiles_early)) != hipSuccess) return fail_hip(c, e, "attract");
        if (ev) (void)hipEventRecord(ev[4], sa);
        if (two && (e = hipEventRecord(c->ev_join, c->stream2)) != hipSuccess) return fail_hip(c, e, "event record");
        return TSNE_OK;
    };
    int rc;
    if (ev) (void)hipEventRecord(ev[0], c->stream);
    // (inside tsne_run the previous update has already left Y in slot order and its bounding box)
    if (!cached && (e = launch_gather_bbox(c, d_Y, c->stream)) != hipSuccess) return fail_hip(c, e, "gather + bbox");
    c->root_fresh = 0;
    if (tiles_early && (e = launch_tree_root(c, c->stream)) != hipSuccess) return fail_hip(c, e, "root square");
    if (two && ((rc = fork(c->ev_fork)) != TSNE_OK || (rc = farpart()) != TSNE_OK)) return rc;
    if ((e = launch_tree_sort(c, c->stream)) != hipSuccess) return fail_hip(c, e, "tree sort");
    if ((e = launch_tree_cells(c, c->stream)) != hipSuccess) return fail_hip(c, e, "tree cells");
    if (ev) (void)hipEventRecord(ev[1], c->stream);
    if (two && ((rc = fork(c->ev_fork2)) != TSNE_OK || (rc = mainpart()) != TSNE_OK)) return rc;
    if ((e = launch_walk(c, c->stream)) != hipSuccess) return fail_hip(c, e, "walk");
    if (ev) (void)hipEventRecord(ev[2], c->stream);
    if (two) {
        if ((e = hipStreamWaitEvent(c->stream, c->ev_join, 0)) != hipSuccess) return fail_hip(c, e, "stream wait");
    } else {
        if ((rc = farpart()) != TSNE_OK || (rc = mainpart()) != TSNE_OK) return rc;
    }
    // Without renumbering, the attractive kernel of the NEXT call visits rows in this call's
    // spatial order (the kernel has finished by now on either stream, so the array is free to
    // overwrite).  With renumbering the slots themselves are ordered and rows go in slot order.
    if (!c->reorder_on &&
        (e = hipMemcpyAsync(c->row_order, c->perm, 4 * (size_t)c->p.n, hipMemcpyDeviceToDevice,
                            c->stream)) != hipSuccess)
        return fail_hip(c, e, "copy row order");
    c->tree_valid = 1;
    return TSNE_OK;
}

// Back to the caller's numbering (slot s = point s): needed before a new P is taken over.
int reset_slot_order(tsne_ctx *c)
{
    if (c->identity) return TSNE_OK;
    const int a = c->cur_state, b = a ^ 1, n = c->p.n;
    hipError_t e;
    if ((e = launch_scatter2(c->uYb[a], c->orig[a], c->uYb[b], n, c->stream)) != hipSuccess ||
        (e = launch_scatter2(c->gainsb[a], c->orig[a], c->gainsb[b], n, c->stream)) != hipSuccess ||
        (e = launch_iota(c->orig[b], n, c->stream)) != hipSuccess ||
        (e = launch_iota(c->row_order, n, c->stream)) != hipSuccess)
        return fail_hip(c, e, "reset slot order");
    c->cur_state = b;
    c->identity = 1;
    c->steps_since_reorder = 0;
    c->arow_valid = 0;
    return TSNE_OK;
}

void free_timing(tsne_ctx *c)
{
    if (!c->tev) return;
    for (int i = 0; i < NEV * c->t_cap; ++i) if (c->tev[i]) (void)hipEventDestroy(c->tev[i]);
    free(c->tev);
    c->tev = nullptr;
    c->t_cap = c->t_used = 0;
}

}  // namespace

extern "C" {

int tsne_default_params(tsne_params *p, int32_t n)
{
    if (!p) return TSNE_EINVAL;
    memset(p, 0, sizeof(*p));
    p->n = n;
    p->theta = 0.5f;
    p->lr = 200.0f;
    p->exaggeration = 12.0f;
    p->exaggeration_iters = 250;
    p->momentum_early = 0.5f;
    p->momentum_late = 0.8f;
    p->momentum_switch_iter = 250;
    p->gain_inc = 0.2f;
    p->gain_dec = 0.8f;
    p->gain_min = 0.01f;
    p->morton_bits = n >= 1 ? std::min(22, (64 - index_bits(n)) / 2) : 22;
    p->leaf_cap = 8;
    p->overlap = 1;
    p->graph_order_iters = 64;
    p->reorder_every = 0;
    p->attract_resident = 1;
    p->walk_resident = 14;
    p->far_tiles = 0;
    p->max_nnz = 0;
    return TSNE_OK;
}

int tsne_workspace_bytes(const tsne_params *p, size_t *bytes)
{
    int rc = check_params(p);
    if (rc != TSNE_OK || !bytes) return TSNE_EINVAL;
    *bytes = carve(nullptr, p, nullptr);
    return TSNE_OK;
}

int tsne_create(tsne_ctx **out, const tsne_params *p, void *stream, void *d_workspace, size_t workspace_bytes)
{
    if (!out) return TSNE_EINVAL;
    *out = nullptr;
    int rc = check_params(p);
    if (rc != TSNE_OK) return rc;
    if (!d_workspace || ((uintptr_t)d_workspace % ALIGN) != 0) return TSNE_EINVAL;
    if (workspace_bytes < carve(nullptr, p, nullptr)) return TSNE_ENOSPC;
    tsne_ctx *c = new (std::nothrow) tsne_ctx();
    if (!c) return TSNE_ENOSPC;
    memset(c, 0, sizeof(*c));
    c->p = *p;
    c->stream = (hipStream_t)stream;
    carve(c, p, (char *)d_workspace);
    c->key_shift = 64 - 2 * p->morton_bits;
    c->reorder_on = (p->reorder_every > 0 || p->graph_order_iters > 0) && p->max_nnz > 0;
    c->identity = 1;
    hipError_t e;
    {
        int dev = 0;
        if ((e = hipGetDevice(&dev)) != hipSuccess ||
            (e = hipDeviceGetAttribute(&c->num_cu, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess ||
            c->num_cu <= 0) {
            tsne_destroy(c);
            return TSNE_EHIP;
        }
    }
    c->sort_items = sort_items(p->n, c->num_cu);
    if (p->overlap) {
        // default priority on purpose; non-blocking so that it does not serialise with stream 0
        if ((e = hipStreamCreateWithFlags(&c->stream2, hipStreamNonBlocking)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&c->ev_fork2, hipEventDisableTiming)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming)) != hipSuccess) {
            tsne_destroy(c);
            return TSNE_EHIP;
        }
    }
    if (p->n <= SMALL_SORT_MAX && (e = small_sort_prepare()) != hipSuccess) {
        tsne_destroy(c);
        return TSNE_EHIP;
    }
    if (c->ft_tiles > 0 &&
        ((e = attract_far_tiled_prepare()) != hipSuccess ||
         (e = hipMemsetAsync(c->ft_cnt, 0, 4 * (size_t)c->ft_tiles, c->stream)) != hipSuccess ||
         (e = hipMemsetAsync(c->ft_acc, 0, 16 * (size_t)p->n, c->stream)) != hipSuccess ||
         (e = hipMemsetAsync(c->ft_meta, 0, 32, c->stream)) != hipSuccess)) {
        tsne_destroy(c);
        return TSNE_EHIP;
    }
    if ((e = hipMemsetAsync(c->status, 0, sizeof(uint32_t), c->stream)) != hipSuccess ||
        (e = hipMemsetAsync(c->ncells, 0, sizeof(uint32_t), c->stream)) != hipSuccess ||
        (e = launch_fill_state(c, c->stream)) != hipSuccess ||
        (e = launch_iota(c->row_order, p->n, c->stream)) != hipSuccess ||
        (e = launch_iota(c->orig[0], p->n, c->stream)) != hipSuccess) {
        tsne_destroy(c);
        return TSNE_EHIP;
    }
    *out = c;
    return TSNE_OK;
}

void tsne_destroy(tsne_ctx *c)
{
    if (!c) return;
    if (c->stream2) { (void)hipStreamSynchronize(c->stream2); (void)hipStreamDestroy(c->stream2); }
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_fork2) (void)hipEventDestroy(c->ev_fork2);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    free_timing(c);
    delete c;
}

int tsne_set_P(tsne_ctx *c, const int32_t *d_row_ptr, const int32_t *d_col, const float *d_val, int64_t nnz)
{
    if (!c) return TSNE_EINVAL;
    if (!d_row_ptr || nnz < 0 || nnz > 0x7FFFFFFFll || (nnz > 0 && (!d_col || !d_val)))
        return fail(c, TSNE_EINVAL, "tsne_set_P: null array or nnz out of range");
    if (c->reorder_on && nnz > c->p.max_nnz) return fail(c, TSNE_ENOSPC, "tsne_set_P: nnz exceeds max_nnz");
    int rc = reset_slot_order(c);
    if (rc != TSNE_OK) return rc;
    c->user_row_ptr = d_row_ptr; c->user_col = d_col; c->user_val = d_val;
    c->nnz = nnz;
    c->arow_valid = 0;
    c->have_P = 1;
    c->ft_far_entries = 0;
    if (c->reorder_on && c->p.graph_order_iters > 0 && nnz > 0) {
        hipError_t e;
        if ((e = launch_graph_order(c, c->stream)) != hipSuccess ||
            (e = launch_reorder(c, c->stream, c->ft_tiles > 0 ? c->p.far_tiles : 1)) != hipSuccess)
            return fail_hip(c, e, "graph order");
        // which kernel takes the far part is settled here, once per P, so that a run is reproducible:
        // later renumberings keep the choice
        c->ft_active = 0;
        if (c->ft_tiles > 0) {
            uint32_t meta_h[5] = {0u, 0u, 0u, 0u, 0u};
            if ((e = hipMemcpyAsync(meta_h, c->ft_meta, sizeof(meta_h), hipMemcpyDeviceToHost, c->stream)) != hipSuccess ||
                (e = hipStreamSynchronize(c->stream)) != hipSuccess)
                return fail_hip(c, e, "graph order");
            c->ft_active = meta_h[0] ? 1 : 0;
            c->ft_far_entries = (int64_t)meta_h[4];
        }
    } else {
        c->ft_active = c->ft_tiles > 0 && c->p.far_tiles == 2;
    }
    return TSNE_OK;
}

int tsne_P_layout(tsne_ctx *c, int64_t *near_entries, int64_t *far_entries)
{
    if (!c) return TSNE_EINVAL;
    if (!c->have_P) return fail(c, TSNE_ESTATE, "tsne_P_layout: no P");
    int64_t near = 0, far = c->nnz;
    if (c->reorder_on && !c->identity) {
        int32_t a = 0, b0 = 0, b1 = 0;
        hipError_t e = hipMemcpyAsync(&a, c->rp_near + c->p.n, 4, hipMemcpyDeviceToHost, c->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(&b0, c->rp_far, 4, hipMemcpyDeviceToHost, c->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(&b1, c->rp_far + c->p.n, 4, hipMemcpyDeviceToHost, c->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
        if (e != hipSuccess) return fail_hip(c, e, "P layout");
        near = a;
        far = (int64_t)b1 - b0;
    }
    if (near_entries) *near_entries = near;
    if (far_entries) *far_entries = far;
    return TSNE_OK;
}

int tsne_init_state(tsne_ctx *c)
{
    if (!c) return TSNE_EINVAL;
    hipError_t e = launch_fill_state(c, c->stream);
    return e == hipSuccess ? TSNE_OK : fail_hip(c, e, "fill state");
}

int tsne_get_state(tsne_ctx *c, float *d_velocity, float *d_gains)
{
    if (!c || !d_velocity || !d_gains) return TSNE_EINVAL;
    const int a = c->cur_state;
    hipError_t e;
    if ((e = launch_scatter2(c->uYb[a], c->orig[a], (float2 *)d_velocity, c->p.n, c->stream)) != hipSuccess ||
        (e = launch_scatter2(c->gainsb[a], c->orig[a], (float2 *)d_gains, c->p.n, c->stream)) != hipSuccess)
        return fail_hip(c, e, "copy state");
    return TSNE_OK;
}

int tsne_set_state(tsne_ctx *c, const float *d_velocity, const float *d_gains)
{
    if (!c || !d_velocity || !d_gains) return TSNE_EINVAL;
    const int a = c->cur_state;
    hipError_t e;
    if ((e = launch_gather2((const float2 *)d_velocity, c->orig[a], c->uYb[a], c->p.n, c->stream)) != hipSuccess ||
        (e = launch_gather2((const float2 *)d_gains, c->orig[a], c->gainsb[a], c->p.n, c->stream)) != hipSuccess)
        return fail_hip(c, e, "copy state");
    return TSNE_OK;
}

namespace {
// One iteration.  cached: Yi / the bounding box were left by the previous call's update (same Y,
// untouched since); keep: leave them for the next call.
int step_impl(tsne_ctx *c, float *d_Y, int32_t iter, bool cached, bool keep)
{
    hipEvent_t *ev = nullptr;      // timed steps: every t_every-th one while slots are left
    if (c->tev && c->t_used < c->t_cap && (c->t_seen++ % c->t_every) == 0) ev = c->tev + NEV * c->t_used;
    const bool use = cached && c->yi_fresh;
    c->yi_fresh = 0;
    int rc = enqueue_forces(c, d_Y, ev, use);
    if (rc != TSNE_OK) return rc;
    const float alpha = iter < c->p.exaggeration_iters ? c->p.exaggeration : 1.0f;
    const float mom = iter < c->p.momentum_switch_iter ? c->p.momentum_early : c->p.momentum_late;
    if (ev) (void)hipEventRecord(ev[8], c->stream);
    // an iteration whose successor reads the embedding from the library's own copy (keep) need not
    // write the caller's array -- unless the slots are about to be renumbered, which starts from it
    const bool renumber_next = c->reorder_on && c->p.reorder_every > 0 && c->steps_since_reorder + 1 >= c->p.reorder_every;
    hipError_t e = launch_update(c, d_Y, alpha, mom, keep ? 1 : 0, (!keep || renumber_next) ? 1 : 0, c->stream);
    if (ev) { (void)hipEventRecord(ev[5], c->stream); c->t_used += 1; }
    if (e != hipSuccess) return fail_hip(c, e, "update");
    c->yi_fresh = keep ? 1 : 0;
    if (c->reorder_on && c->p.reorder_every > 0 && ++c->steps_since_reorder >= c->p.reorder_every) {
        c->steps_since_reorder = 0;
        c->yi_fresh = 0;      // the slots are renumbered: Yi is stale
        if ((e = launch_reorder(c, c->stream, c->ft_active ? 2 : 1)) != hipSuccess) return fail_hip(c, e, "reorder");
    }
    return TSNE_OK;
}
}  // namespace

int tsne_step(tsne_ctx *c, float *d_Y, int32_t iter)
{
    if (!c || !d_Y || iter < 0) return TSNE_EINVAL;
    if (!c->have_P) return fail(c, TSNE_ESTATE, "tsne_step: no P (call tsne_set_P first)");
    return step_impl(c, d_Y, iter, false, false);
}

int tsne_timing_begin(tsne_ctx *c, int32_t max_steps) { return tsne_timing_begin_every(c, max_steps, 1); }

int tsne_timing_begin_every(tsne_ctx *c, int32_t max_steps, int32_t every)
{
    if (!c || max_steps < 1 || max_steps > (1 << 20) || every < 1) return TSNE_EINVAL;
    free_timing(c);
    c->t_every = every;
    c->t_seen = 0;
    c->tev = (hipEvent_t *)calloc((size_t)NEV * max_steps, sizeof(hipEvent_t));
    if (!c->tev) return TSNE_ENOSPC;
    c->t_cap = max_steps;
    for (int i = 0; i < NEV * max_steps; ++i) {
        hipError_t e = hipEventCreate(&c->tev[i]);
        if (e != hipSuccess) { free_timing(c); return fail_hip(c, e, "event create"); }
    }
    return TSNE_OK;
}

int tsne_timing_end(tsne_ctx *c, int32_t *steps, float ms[4])
{
    if (!c) return TSNE_EINVAL;
    if (!c->tev) return fail(c, TSNE_ESTATE, "tsne_timing_end: timing was not begun");
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e == hipSuccess && c->stream2) e = hipStreamSynchronize(c->stream2);
    if (e != hipSuccess) return fail_hip(c, e, "sync");
    double acc[4] = {0, 0, 0, 0};
    // tree, walk, attraction (main piece + early piece), update
    static const int from[5] = {0, 1, 3, 8, 6}, to[5] = {1, 2, 4, 5, 7}, into[5] = {0, 1, 2, 3, 2};
    for (int s = 0; s < c->t_used; ++s)
        for (int q = 0; q < 5; ++q) {
            float t = 0.f;
            e = hipEventElapsedTime(&t, c->tev[NEV * s + from[q]], c->tev[NEV * s + to[q]]);
            if (e != hipSuccess) { free_timing(c); return fail_hip(c, e, "event elapsed"); }
            acc[into[q]] += t;
        }
    if (steps) *steps = c->t_used;
    if (ms) for (int q = 0; q < 4; ++q) ms[q] = c->t_used ? (float)(acc[q] / c->t_used) : 0.f;
    free_timing(c);
    return TSNE_OK;
}

int tsne_status(tsne_ctx *c, uint32_t *status)
{
    if (!c || !status) return TSNE_EINVAL;
    hipError_t e = hipMemcpyAsync(status, c->status, sizeof(uint32_t), hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    return e == hipSuccess ? TSNE_OK : fail_hip(c, e, "status");
}

int tsne_run(tsne_ctx *c, float *d_Y, int32_t iter0, int32_t n_iter)
{
    if (!c || !d_Y || iter0 < 0 || n_iter < 0) return TSNE_EINVAL;
    if (!c->have_P) return fail(c, TSNE_ESTATE, "tsne_run: no P (call tsne_set_P first)");
    // Between the iterations of one call nobody else touches Y, so every update hands the next
    // iteration the embedding in slot order and its bounding box.
    for (int32_t it = iter0; it < iter0 + n_iter; ++it) {
        const bool cached = it > iter0, keep = it + 1 < iter0 + n_iter;
        int rc = step_impl(c, d_Y, it, cached, keep);
        if (rc != TSNE_OK) { c->yi_fresh = 0; return rc; }
    }
    c->yi_fresh = 0;
    uint32_t st = 0;
    int rc = tsne_status(c, &st);
    if (rc != TSNE_OK) return rc;
    if (st) {
        snprintf(c->err, sizeof(c->err), "device status 0x%x", st);
        return TSNE_ENUM;
    }
    return TSNE_OK;
}

int tsne_gradient(tsne_ctx *c, const float *d_Y, float *d_attr, float *d_rep, double *d_Z)
{
    if (!c || !d_Y) return TSNE_EINVAL;
    if (!c->have_P) return fail(c, TSNE_ESTATE, "tsne_gradient: no P (call tsne_set_P first)");
    int rc = enqueue_forces(c, d_Y, nullptr);
    if (rc != TSNE_OK) return rc;
    const uint32_t *orig = c->orig[c->cur_state];
    hipError_t e = hipSuccess;
    if (d_attr) e = launch_scatter2(c->A, orig, (float2 *)d_attr, c->p.n, c->stream);
    if (e == hipSuccess && d_rep) e = launch_scatter2(c->R, orig, (float2 *)d_rep, c->p.n, c->stream);
    if (e == hipSuccess && d_Z) e = hipMemcpyAsync(d_Z, c->Z, 8, hipMemcpyDeviceToDevice, c->stream);
    return e == hipSuccess ? TSNE_OK : fail_hip(c, e, "copy forces");
}

int tsne_export_tree(tsne_ctx *c, uint64_t *d_keys, int32_t *d_perm, int32_t cap_cells, int32_t *d_depth,
                     int32_t *d_lo, int32_t *d_hi, int32_t *d_leaf, float *d_com, float *d_root, int32_t *n_cells)
{
    if (!c || cap_cells < 0) return TSNE_EINVAL;
    if (!c->tree_valid) return fail(c, TSNE_ESTATE, "tsne_export_tree: no tree built yet");
    hipError_t e = hipSuccess;
    if (d_keys || d_perm) e = launch_export_order(c, d_keys, d_perm, c->stream);
    if (e == hipSuccess && d_root) e = hipMemcpyAsync(d_root, c->root, 12, hipMemcpyDeviceToDevice, c->stream);
    if (e == hipSuccess) e = launch_export_cells(c, cap_cells, d_depth, d_lo, d_hi, d_leaf, d_com, c->stream);
    uint32_t m = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&m, c->ncells, 4, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return fail_hip(c, e, "export tree");
    if (n_cells) *n_cells = (int32_t)m;
    if ((int64_t)m > (int64_t)c->cap_cells) return fail(c, TSNE_ENUM, "tree needed more cells than the workspace holds");
    if ((int64_t)m > (int64_t)cap_cells && (d_depth || d_lo || d_hi || d_leaf || d_com))
        return fail(c, TSNE_ENOSPC, "tsne_export_tree: cap_cells too small");
    return TSNE_OK;
}

int tsne_kl(tsne_ctx *c, const float *d_Y, double *kl)
{
    if (!c || !d_Y || !kl) return TSNE_EINVAL;
    if (!c->have_P) return fail(c, TSNE_ESTATE, "tsne_kl: no P");
    hipError_t e = launch_kl(c, d_Y, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(kl, c->kl_part, 8, hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    return e == hipSuccess ? TSNE_OK : fail_hip(c, e, "kl");
}

const char *tsne_strerror(int code)
{
    switch (code) {
    case TSNE_OK: return "ok";
    case TSNE_EINVAL: return "invalid argument";
    case TSNE_ENOSPC: return "workspace or output capacity too small";
    case TSNE_EHIP: return "HIP runtime error";
    case TSNE_ESTATE: return "call out of order";
    case TSNE_ENUM: return "numerical trouble reported by the device";
    default: return "unknown error";
    }
}

const char *tsne_last_error(const tsne_ctx *c) { return c ? c->err : ""; }

}  // extern "C"
