// Internal declarations shared by the HIP translation units of the library.
// gfx950 only: wavefronts are 64 lanes wide and the code relies on it.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tsne.h"

#define TSNE_NONE 0xFFFFFFFFu
#define WAVE 64

// One quad-tree cell, 32 bytes so that a lane fetches it with two 16-byte loads.
// Cells are stored in depth-first pre-order; the first child of cell c is c + 1.
struct __align__(32) Cell {
    float cx, cy;      // centre of mass (Eq. (15): y_cell)
    uint32_t cnt;      // N_cell
    uint32_t meta;     // depth | (leaf << 8)
    uint32_t lo;       // first member position in the spatial order
    uint32_t c1, c2, c3;  // 2nd..4th existing child, TSNE_NONE if absent
};

struct ScanPart {
    double sx, sy;
    uint32_t cnt;
    uint32_t pad;
};

// Tiling constants that host and device must agree on.
constexpr int RADIX_BITS = 11;           // digit width of the radix sort
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_THREADS = 512;
constexpr int SORT_TILE_MIN = SORT_THREADS * 8;   // smallest tile of the sort (words per thread: 8, 10 or 12)
constexpr int MAX_GRID_BITS = 24;        // a float has 24 significant bits
constexpr int SMALL_SORT_MAX = 8192;  // up to here one workgroup finds root, keys and order in LDS
constexpr int LEVEL_THREADS = 256;
constexpr int LEVEL_ITEMS = 4;
constexpr int LEVEL_TILE = LEVEL_THREADS * LEVEL_ITEMS;
constexpr int BBOX_MAX_BLOCKS = 1024;
constexpr int WALK_COUNTERS = 16;        // work counters of the resident walk (a power of two)
constexpr int ATTRACT_BAND = 1280;       // half width of the near part of the renumbered P
constexpr int ATTRACT_ROWS = 512;        // rows the attraction kernel's window of Y advances by
constexpr int ATTRACT_RING = ATTRACT_ROWS + 2 * ATTRACT_BAND;   // points in that window (a ring in LDS)
static_assert(ATTRACT_RING * 8 <= 65536, "ring offsets are stored in 16 bits");
constexpr int ATTRACT_CHUNK = 32;        // near rows are padded to a multiple of this many entries
constexpr int ATTRACT_SLACK = 64;        // entries readable past the end of col_s / val_s
constexpr int ATTRACT_MAX_PARTS = 16384; // most resident workgroups of the attraction kernel
constexpr int FT_ROWS = 6144;            // rows of a tile of the bucketed copy of the far part
constexpr int FT_COLS = 2048;            // columns of such a tile
constexpr int FT_MIN_POINTS = 3 << 16;   // fewest points for which the tiles are chosen automatically
constexpr int64_t FT_MAX_TILES = (int64_t)1 << 27;

struct tsne_ctx {
    tsne_params p;
    hipStream_t stream;
    hipStream_t stream2;
    int num_cu;                    // compute units of the current device
    hipEvent_t ev_fork, ev_fork2, ev_join;
    int have_P, tree_valid;
    int t_every, t_seen;           // timing: every t_every-th step is timed; steps seen since timing began
    // P in the caller's numbering (borrowed)
    const int32_t *user_row_ptr, *user_col;
    const float *user_val;
    int64_t nnz;
    // slot order: slot s holds original point orig[cur_state][s]; velocity and gains live in slot order
    int reorder_on, cur_state, steps_since_reorder, identity;
    uint32_t *orig[2], *inv;     // inv: caller's index -> slot
    // P in slot numbering, split by distance from the diagonal (valid while !identity): entries
    // with |column - row| <= ATTRACT_BAND form the near part (rows padded with zero weights to a
    // multiple of ATTRACT_CHUNK entries, so every row starts on a 128-byte line and no line is
    // shared between rows), the others the far part.  Values of both live in val_s, the far part
    // after the near part (rp_far holds positions in val_s).  A near column is stored as the
    // 16-bit byte offset of its point in the LDS ring of Y that the attraction kernel keeps
    // (8 (column mod ATTRACT_RING)); far columns are slot numbers, col_far[j - rp_far[0]].
    int32_t *rp_near, *rp_far, *col_far, *len_near, *len_far;
    uint16_t *col_near;
    uint32_t *far_rows, *far_count;   // the rows that have a far part (any order), and how many
    float2 *Afar;                     // their far sums, by row
    float *val_s;
    // the far part once more, bucketed by tiles of FT_ROWS x FT_COLS (row tile major); an entry is
    // (column, row within the row tile, value), in any order inside its tile
    int64_t ft_tiles;                 // number of tiles, 0 if the context has no room for them
    int64_t ft_far_entries;           // entries of the far part when P was set (0: not known)
    int ft_nct;                       // column tiles per row
    uint32_t *ft_cnt;                 // per tile: entries not yet placed (0 outside ft_fill_k)
    int32_t *ft_ptr;                  // per tile: first entry (+ end)
    int32_t *ft_col;
    uint16_t *ft_row;
    float *ft_val;
    double *ft_acc;                   // row sums in fixed point (integer-valued doubles), (x, y) per row; zero between steps
    int ft_active;                    // the tiles are in use (decided at tsne_set_P, kept through later renumberings)
    uint32_t *ft_meta;                // [0] tiles in use, [1] largest P value (bits), [2] longest far row, [4] entries of the far part
    float2 *Yi, *uYb[2], *gainsb[2];
    // workspace carve-up
    float4 *bbox_part;   // (min, max) pairs of the bounding box, one per workgroup of the kernel that made them
    int bbox_nparts;     // how many pairs are valid
    int root_fresh;      // the root square of this step is already in place (launch_tree_root)
    int yi_fresh;        // Yi and bbox_part already hold the embedding of the next step (left by update_k)
    float4 *root;        // x0, y0, W, S
    uint32_t *status;    // device status word
    uint32_t *ncells;    // device cell count
    // the sort works on one 64-bit word per point: (grid key << key_shift) | slot, key_shift = 64 - 2 morton_bits,
    // so that the order of the words is the order by (key, slot) and no separate index array travels along
    uint64_t *words[2];
    int key_shift;
    uint32_t *perm;      // spatial order: position p holds slot perm[p] (written with the sorted points)
    int32_t *arow;              // first row of each resident workgroup of the attraction kernel (+ end)
    int arow_valid;             // arow matches the current near part
    uint32_t *row_order; // order in which the attractive kernel visits the rows (an earlier spatial order)
    uint32_t *hist, *dtot;
    float2 *Ys;
    uint16_t *lev;
    ScanPart *part;
    uint32_t *cellseq;
    double2 *ps;
    Cell *cells;
    int32_t cap_cells;
    uint32_t *cell_p;      // position and depth of every cell, by cell number
    uint8_t *cell_t;
    uint32_t *walk_counter; // work counter of the resident walk (zeroed by the tree build)
    uint32_t *big_count;   // cells too large for the in-LDS searches, finished by a second kernel
    uint2 *big_list;
    int32_t big_cap;
    float2 *R, *A;
    double *zpart, *Z;
    double *kl_part;
    int sorted_buf;      // which of words[] holds the sorted result
    int sort_items;      // words per thread of the sort's tiles (sort_items())
    // optional per-phase timing: 9 events per armed step
    hipEvent_t *tev;
    int t_cap, t_used;
    char err[256];
};

// ---- launchers (each enqueues on the given stream and returns the launch error) ----
inline bool ft_possible(const tsne_params *p)
{
    const int64_t nrt = ((int64_t)p->n + FT_ROWS - 1) / FT_ROWS, nct = ((int64_t)p->n + FT_COLS - 1) / FT_COLS;
    return p->far_tiles != 1 && nrt * nct <= FT_MAX_TILES;
}
hipError_t attract_far_tiled_prepare();   // once per process, before the first launch
hipError_t small_sort_prepare();          // likewise

// inverted-file neighbour search (ivf.hip); return a tsne_error
size_t ivf_workspace(int n, int d, int k, int nlist, int tau);
int ivf_train_device(const float *X, int n, int d, int nlist, int iters, float *C, void *ws, size_t ws_bytes, hipStream_t s);
// the same for long rows on the matrix-core tiles of the exact search (build_p.hip); probe, lorder, cellptr on the device.
// ivf_tiles_workspace: bytes for ivf_probe_tiles and (k > 0) ivf_search_tiles, or 0 if the sizes are beyond them.
size_t ivf_tiles_workspace(int n, int d, int k, int nlist, int tau);
int ivf_probe_tiles(const float *X, int n, int d, const float *C, int nlist, int tau, int m, int32_t *probe, void *ws,
                    size_t ws_bytes, hipStream_t s, int reuse_queries);
int ivf_search_tiles(const float *X, int n, int d, int k, int nlist, int tau, const int32_t *probe, const int *lorder,
                     const int *cellptr, int max_list, long long max_cand, int32_t *knn_idx, double *knn_d2, void *ws,
                     size_t ws_bytes, hipStream_t s);
int ivf_knn_device(const float *X, int n, int d, const float *C, int nlist, int tau, int k, int32_t *knn_idx,
                   double *knn_d2, void *ws, size_t ws_bytes, hipStream_t s);
hipError_t launch_gather_bbox(tsne_ctx *c, const float *d_Y, hipStream_t s);
hipError_t launch_tree_root(tsne_ctx *c, hipStream_t s);
hipError_t launch_tree_sort(tsne_ctx *c, hipStream_t s);
hipError_t launch_tree_cells(tsne_ctx *c, hipStream_t s);
hipError_t launch_walk(tsne_ctx *c, hipStream_t s);
// the far part of the renumbered P (no-op otherwise); tiles: the bucketed copy is summed here rather than in launch_attract_main
hipError_t launch_attract_far(tsne_ctx *c, hipStream_t s, bool tiles);
hipError_t launch_attract_main(tsne_ctx *c, hipStream_t s, bool tiles);
hipError_t launch_update(tsne_ctx *c, float *d_Y, float alpha, float momentum, int keep, int write_user,
                         hipStream_t s);
hipError_t launch_reorder(tsne_ctx *c, hipStream_t s, int tiles_mode);   // tiles_mode: 0 decide, 1 rows, 2 tiles
hipError_t launch_graph_order(tsne_ctx *c, hipStream_t s);   // leaves the order in c->perm
// stable sort of words[0] on bits [lo, lo + nbits); result in words[sorted_buf].  hist0: the digit counts of the
// first pass are already in c->hist (left by the kernel that wrote the words)
int sort_items(int n, int num_cu);
hipError_t launch_sort(tsne_ctx *c, int lo, int nbits, bool hist0, hipStream_t s);
hipError_t launch_unpack_perm(tsne_ctx *c, hipStream_t s);   // c->perm = low 32 bits of words[sorted_buf] (the graph order's words)
hipError_t launch_scatter2(const float2 *in, const uint32_t *orig, float2 *out, int n, hipStream_t s);
hipError_t launch_gather2(const float2 *in, const uint32_t *orig, float2 *out, int n, hipStream_t s);
hipError_t launch_export_order(tsne_ctx *c, uint64_t *d_keys, int32_t *d_perm, hipStream_t s);
hipError_t launch_fill_state(tsne_ctx *c, hipStream_t s);
hipError_t launch_iota(uint32_t *a, int n, hipStream_t s);
hipError_t launch_export_cells(tsne_ctx *c, int32_t cap, int32_t *depth, int32_t *lo, int32_t *hi,
                               int32_t *leaf, float *com, hipStream_t s);
hipError_t launch_kl(tsne_ctx *c, const float *d_Y, hipStream_t s);  // result in c->kl_part[0]

// ---- wave helpers ----
// One axis of a launch holds fewer than 2^32 work-items: the dispatch packet counts them in 32 bits, and a larger
// product of workgroups and workgroup size wraps without any error.  Launches with one work-item (or a few) per
// element of a large array therefore spread their workgroups over two axes, and the kernel takes its element
// number from global_index().  Along x at most 2^23 workgroups of at most 256, so any count below 2^31 stays on x.
inline dim3 wide_grid(size_t items, int per = 256)
{
    const size_t nb = (items + (size_t)per - 1) / (size_t)per, gx = (size_t)1 << 23;
    if (nb <= gx) return dim3((unsigned)(nb > 0 ? nb : 1));
    return dim3((unsigned)gx, (unsigned)((nb + gx - 1) / gx));
}
__device__ __forceinline__ size_t global_block() { return (size_t)blockIdx.y * gridDim.x + blockIdx.x; }
__device__ __forceinline__ size_t global_index()
{
    return ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (WAVE - 1)); }

__device__ __forceinline__ uint64_t lanemask_lt()
{
    return (1ull << lane_id()) - 1ull;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

__device__ __forceinline__ float wave_min(float v)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, WAVE));
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}

// Data-parallel primitive moves between lanes (no LDS traffic).  CTRL: 0xB1 swaps neighbours,
// 0x4E swaps pairs inside every four lanes, 0x141 mirrors every eight lanes, 0x00 copies the
// first lane of every four, 0x114 shifts by four lanes inside every sixteen.
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) { return __int_as_float(dpp_i<CTRL>(__float_as_int(v))); }
// sum over every aligned group of eight lanes, delivered to all eight; all lanes must be active
__device__ __forceinline__ float sum8(float v)
{
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    return v;
}
// the same for groups of four lanes
__device__ __forceinline__ float sum4(float v)
{
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    return v;
}
// value of the first lane of every aligned group of four lanes
__device__ __forceinline__ int first4(int v) { return dpp_i<0x00>(v); }

// Exclusive prefix sum over the 64 lanes; *total receives the wave sum.  All lanes must be
// active.  Log-step shifts inside every row of 16 lanes (0x111, 0x112, 0x114, 0x118: shift right
// by 1, 2, 4, 8 with zero fill), then the last lane of a row is added to the next row (0x142,
// rows 1 and 3) and lane 31 to the upper half (0x143, rows 2 and 3).
__device__ __forceinline__ int wave_excl_scan(int v, int *total)
{
    int inc = v;
    inc += __builtin_amdgcn_update_dpp(0, inc, 0x111, 0xF, 0xF, true);
    inc += __builtin_amdgcn_update_dpp(0, inc, 0x112, 0xF, 0xF, true);
    inc += __builtin_amdgcn_update_dpp(0, inc, 0x114, 0xF, 0xF, true);
    inc += __builtin_amdgcn_update_dpp(0, inc, 0x118, 0xF, 0xF, true);
    inc += __builtin_amdgcn_update_dpp(0, inc, 0x142, 0xA, 0xF, false);
    inc += __builtin_amdgcn_update_dpp(0, inc, 0x143, 0xC, 0xF, false);
    *total = __builtin_amdgcn_readlane(inc, WAVE - 1);
    return inc - v;
}
