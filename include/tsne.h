/*
 * tsne.h -- C ABI of the MI355X (gfx950) Barnes-Hut t-SNE library.
 *
 * The library implements the per-iteration gradient step of Barnes-Hut t-SNE as
 * laid out in Algorithm 1 of "t-SNE-CUDA" (arXiv 1807.11824): tree build,
 * repulsive forces with the Z estimate, attractive forces over the sparse P,
 * and the update of the embedding -- plus the one-off construction of P.
 *
 * Conventions
 *  - Every pointer named d_* is a DEVICE pointer into memory the caller owns
 *    (e.g. a torch tensor's data_ptr()); every other pointer is a HOST pointer.
 *  - The library allocates no device memory: the caller passes one workspace of
 *    at least tsne_workspace_bytes() / tsne_build_P_workspace_bytes() bytes,
 *    256-byte aligned, which must stay alive while the context is in use.
 *  - All work is enqueued on the caller's HIP stream (`stream` is a hipStream_t
 *    passed as void*; NULL = the default stream).  tsne_step() and
 *    tsne_gradient() never synchronise the host; tsne_run(), tsne_status(),
 *    tsne_kl() and tsne_build_P() do.
 *  - Arguments are validated on the host before anything is enqueued.  Every
 *    function returns TSNE_OK (0) or a negative tsne_error; nothing aborts.
 *  - One context must not be used from two threads at once.
 */
#ifndef TSNE_H
#define TSNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TSNE_OK = 0,
    TSNE_EINVAL = -1,  /* bad argument (null pointer, size or parameter out of range) */
    TSNE_ENOSPC = -2,  /* workspace or output capacity too small */
    TSNE_EHIP = -3,    /* a HIP call failed; see tsne_last_error() */
    TSNE_ESTATE = -4,  /* call out of order (e.g. tsne_step before tsne_set_P) */
    TSNE_ENUM = -5     /* numerical trouble reported by the device; see tsne_status() */
} tsne_error;

/* Bits of the device status word returned by tsne_status(). */
#define TSNE_STATUS_NONFINITE 1u     /* a coordinate of Y was NaN or infinite */
#define TSNE_STATUS_CELL_OVERFLOW 2u /* the quad tree needed more cells than the workspace holds */
#define TSNE_STATUS_WALK_OVERFLOW 4u /* internal stack / list bound hit during the tree walk */

/* The wavefront width: points are walked through the tree in groups of this
 * many consecutive positions of the spatial order, all taking the same
 * accept / open decisions (Sec. III-C, last paragraph: divergence-free walk). */
#define TSNE_GROUP 64

typedef struct {
    int32_t n;                    /* number of points, 1 .. 2^27 */
    float theta;                  /* Eq. (14) threshold; 0 <= theta <= 0.7; 0 = all pairs */
    float lr;                     /* learning rate (200) */
    float exaggeration;           /* factor on the attractive term early on (12) */
    int32_t exaggeration_iters;   /* iterations [0, this) are exaggerated (250) */
    float momentum_early;         /* 0.5 */
    float momentum_late;          /* 0.8 */
    int32_t momentum_switch_iter; /* 250 */
    float gain_inc;               /* 0.2 */
    float gain_dec;               /* 0.8 */
    float gain_min;               /* 0.01 */
    int32_t morton_bits;          /* grid bits per axis = maximum tree depth, 1..24, and
                                     2 morton_bits + ceil(log2 n) <= 64 (a point's grid key and its number share a
                                     64-bit word in the sort).  (the smaller of 22 and (64 - ceil(log2 n)) / 2:
                                     21 at n = 1.28M; late in a run whole clusters are smaller than 2^-16 of the
                                     embedding's extent and only a deeper grid splits them) */
    int32_t leaf_cap;             /* a cell with at most this many points is a leaf, >= 1 (8) */
    int32_t overlap;              /* 1: the attractive forces run on a second stream, the entries far from the
                                     diagonal beside the tree build and the streaming part beside the tree walk;
                                     0: everything on one stream.  (1) */
    int32_t graph_order_iters;    /* > 0 (and max_nnz > 0): at tsne_set_P the library renumbers its private
                                     copy of the points and of P so that points that are neighbours in P get
                                     nearby numbers: a seeded pseudo-random value per point is averaged over
                                     the P-neighbourhood this many times and the points are sorted by it.
                                     The sparsity pattern becomes banded, so the y_j gathers of Eq. (5) stay
                                     on chip.  Nothing the method computes changes except float rounding and
                                     the order of points with equal grid keys.  (64) */
    int32_t reorder_every;        /* > 0 (and max_nnz > 0): additionally renumber along the current spatial
                                     order of the embedding every this many steps.  (0 = never) */
    int32_t attract_resident;     /* resident workgroups (512 lanes) of the streaming attraction kernel per
                                     compute unit; each works through a contiguous share of the rows.
                                     0 = library's choice.  (1) */
    int32_t walk_resident;        /* > 0: the tree walk runs as this many resident waves per compute unit that
                                     take groups of points from a counter, so that walk and attraction hold
                                     fixed shares of every compute unit; used when there are more groups than
                                     resident waves.  0 = one wave per group.  (14) */
    int32_t far_tiles;            /* how the entries of the renumbered P that lie far from the diagonal are
                                     summed.  1: one row at a time.  2: from a copy bucketed by 6144-row x
                                     2048-column tiles, row sums kept in fixed point (every addition exact, so
                                     the result does not depend on the order of the entries).  0: chosen at
                                     tsne_set_P: tiles if the far part holds at least half of the entries and
                                     n >= 196,608, rows otherwise; kept through later renumberings.  (0) */
    int64_t max_nnz;              /* capacity for the private, renumbered copy of P: the workspace grows by
                                     20 bytes per entry plus 202 bytes per point (rows are padded) plus 8 bytes
                                     per pair of a 6144-row and a 2048-column tile (n^2 / (3 x 2^22)).  0 disables
                                     renumbering; P is then only borrowed and a stop/resume is bitwise
                                     reproducible.  With renumbering a row of the attractive sum is added up
                                     as (entries near the diagonal) + (the others): deterministic, equal to
                                     the plain order up to rounding. */
} tsne_params;

typedef struct tsne_ctx tsne_ctx; /* opaque, host side, owned by the library */

/* Fills *p with the defaults quoted above for n points (max_nnz = 0: set it to the entry count of P,
 * at most 2 n k, to enable renumbering). */
int tsne_default_params(tsne_params *p, int32_t n);

/* Bytes of device workspace a context with these parameters needs (upper bound). */
int tsne_workspace_bytes(const tsne_params *p, size_t *bytes);

/* Creates a context.  d_workspace: device memory, >= tsne_workspace_bytes(), 256-byte aligned;
 * the optimiser state (velocity, gains) lives inside it.  The context starts with velocity 0,
 * gains 1 and no P. */
int tsne_create(tsne_ctx **out, const tsne_params *p, void *stream, void *d_workspace, size_t workspace_bytes);
void tsne_destroy(tsne_ctx *ctx);

/*
 * Alg. 1 lines 1-2: affinities.  For every row of X (n x d, row-major float, device) the exact k
 * nearest neighbours under squared Euclidean distance (Sec. III-B; self excluded, ordered by
 * (distance, index)), then Eq. (1) restricted to those neighbours with sigma_i set so that the
 * row's entropy is ln(perplexity), then p_ij = (p_j|i + p_i|j) / 2N stored as CSR with ascending
 * columns (at most 2 n k entries).
 * Outputs (device, caller-owned): d_row_ptr[n+1], d_col[cap_nnz], d_val[cap_nnz];
 * cap_nnz >= 2*n*k always suffices.  *nnz (host) receives the entry count.
 * Optional outputs (may be NULL): d_knn_idx[n*k] neighbour indices, d_knn_d2[n*k] squared distances.
 * *n_unconverged (host, may be NULL) receives the number of rows whose entropy could not be
 * brought within 1e-5 of the target (e.g. all neighbours equidistant).
 * X must be finite with |x| < 1e38.  Candidate neighbours are found with reduced-precision products
 * (each value, minus its column's mean, as two bf16 parts; rows of 256 and more coordinates first as one
 * half-precision value), every row's list is then re-ranked in double precision from X itself and checked
 * against a bound on the candidate search's error; rows that cannot be certified go on to the next finer
 * search and finally (ties at the k-th distance) are redone exactly against all n rows, 2k rows a launch, so
 * the lists do not depend on the reduced precision.
 * Workspace: about 4 n (d rounded up to 32) bytes for the split copy of X (half as much again for rows of
 * 256 and more coordinates), 20 n k for neighbour lists and probabilities, 16 n k for sorting, and
 * 8 * 65536 * (k' + 4160) with k' = k + max(k/2, 32) for the candidate buffers
 * (tsne_build_P_workspace_bytes() gives the exact figure).
 * Limits: k' <= 1920, d <= 4096, 2 n k < 2^31.
 * Synchronises the stream before returning.
 */
int tsne_build_P_workspace_bytes(int32_t n, int32_t d, int32_t k, size_t *bytes);
int tsne_build_P(const float *d_X, int32_t n, int32_t d, float perplexity, int32_t k,
                 int32_t *d_row_ptr, int32_t *d_col, float *d_val, int64_t cap_nnz, int64_t *nnz,
                 int32_t *d_knn_idx, float *d_knn_d2, int32_t *n_unconverged,
                 void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Sec. III-B, Eq. (8)-(11): approximate neighbours from an inverted file.  The coarse quantiser q1 is the
 * nearest of nlist centroids (index of the lowest among equals); a query looks at the tau lists whose
 * centroids are nearest to it (Eq. 10) and keeps the k nearest of the points stored in them (Eq. 11).
 * Here the second-stage code q2 of Eq. (8) is the identity: list entries are compared by their exact squared
 * distance (a "flat" inverted file), so the only approximation is in which lists are looked at
 * (tsne_ivfpq_* below: the product-quantised second stage).
 * All decisions are taken on squared distances accumulated in double precision from the float inputs,
 * ties towards the lower index; the lists returned are those of the definition.
 *
 * tsne_ivf_train: k-means (Lloyd) for the centroids, as the paper trains them.  Start: of the sample of
 *   m = min(n, 8 nlist) rows floor(j n / m) the first, then nlist - 1 times the sample row farthest from
 *   those taken so far (lowest j among equals), which puts a centroid into every well separated cluster
 *   before any gets a second one.  Then `iters` rounds, on the min(n, 256 nlist) rows floor(i n / m), of
 *   (assign every row to its nearest centroid, move every centroid to the mean of its rows; a centroid
 *   without rows stays).  d_centroids: nlist x d floats
 *   (device, caller-owned, written).  X must be finite with |x| < 1e38.
 * tsne_ivf_knn: neighbour lists of every row of X (self excluded, ordered by (distance, index)) from
 *   given centroids.  d_knn_idx: n x k int32, d_knn_d2: n x k doubles (device, caller-owned).
 *   Returns TSNE_ENUM if some row finds fewer than k other points in its tau lists (raise tau or lower
 *   nlist), TSNE_ENOSPC if one row's candidates do not fit the workspace's distance scratch.
 * Workspace (tsne_ivf_workspace_bytes; use the figure for the largest tau to be passed): 8 n d bytes for
 *   the copy of X grouped by list, 4 n tau, and a scratch of min(8 GiB, 4 n min(n, 4096)) bytes for one
 *   float per (query, candidate); more workspace than asked for is used (up to 8 GiB of scratch) to take
 *   more queries per pass.  Rows of more than 64 coordinates are searched on the matrix cores (candidates from
 *   tiles of split values, exact re-rank, an exact pass where the re-rank cannot vouch for the result): the
 *   figure then also holds a split copy of X (4 n d bytes) and 8 (k + 4176) bytes per query of a pass of 131,072.
 * Limits: nlist <= min(n, 65536), tau <= min(nlist, 32), k <= 1920, d <= 4096, n tau < 2^31.
 * Both calls synchronise the stream before returning.
 */
int tsne_ivf_workspace_bytes(int32_t n, int32_t d, int32_t k, int32_t nlist, int32_t tau, size_t *bytes);
int tsne_ivf_train(const float *d_X, int32_t n, int32_t d, int32_t nlist, int32_t iters, float *d_centroids,
                   void *d_workspace, size_t workspace_bytes, void *stream);
int tsne_ivf_knn(const float *d_X, int32_t n, int32_t d, const float *d_centroids, int32_t nlist, int32_t tau,
                 int32_t k, int32_t *d_knn_idx, double *d_knn_d2, void *d_workspace, size_t workspace_bytes,
                 void *stream);

/*
 * Sec. III-B, Eq. (8) and (11): the product-quantised second stage.  A point y of list c = q1(y) is stored as m code
 * bytes: its residual y - c (one float subtraction per coordinate) is cut into m sub-vectors of d / m coordinates
 * and each is replaced by the index of the nearest of ksub centroids of that sub-vector's own quantiser (squared
 * distance in double, lowest index among equals); q(y) = c + the m centroids.  A query compares itself with the
 * codes of the points in its tau lists: |x - q(y)|^2 = sum over the sub-vectors j, in order, of
 * sum_t ((x_t - c_t) - codebook[j][code_j][t])^2, every operation in double and none fused; the k smallest by
 * (that value, index) are returned together with those values.
 *
 * tsne_ivfpq_train: the m codebooks.  Sub-quantiser j is tsne_ivf_train's k-means (same start, same sample
 *   rule, `iters` rounds) with ksub centroids on the j-th sub-vectors of the residuals of all rows.
 *   d_codebooks: m x ksub x (d / m) floats (device, caller-owned, written).
 * tsne_ivfpq_knn: codes of all rows, then the search.  d_knn_idx: n x k int32, d_knn_d2: n x k doubles (the
 *   distances to the codes).  Errors as tsne_ivf_knn.
 * Limits: those of tsne_ivf_knn; d a multiple of m; ksub <= min(n, 256).
 * Both calls synchronise the stream before returning.
 */
int tsne_ivfpq_workspace_bytes(int32_t n, int32_t d, int32_t k, int32_t nlist, int32_t tau, int32_t m, int32_t ksub,
                               size_t *bytes);
int tsne_ivfpq_train(const float *d_X, int32_t n, int32_t d, const float *d_centroids, int32_t nlist, int32_t m,
                     int32_t ksub, int32_t iters, float *d_codebooks, void *d_workspace, size_t workspace_bytes,
                     void *stream);
int tsne_ivfpq_knn(const float *d_X, int32_t n, int32_t d, const float *d_centroids, int32_t nlist,
                   const float *d_codebooks, int32_t m, int32_t ksub, int32_t tau, int32_t k, int32_t *d_knn_idx,
                   double *d_knn_d2, void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * tsne_build_P with the neighbours of Sec. III-B's approximate search instead of the exact ones:
 * tsne_ivf_train (nlist centroids, kmeans_iters rounds; nlist = 0 takes the paper's sqrt(n)), tsne_ivf_knn
 * (tau lists per query), then Eq. (1) and the symmetric CSR exactly as in tsne_build_P.  pq_m > 0 takes the
 * product-quantised second stage instead (tsne_ivfpq_train with pq_m sub-vectors of d / pq_m coordinates, 256
 * centroids each, kmeans_iters rounds; tsne_ivfpq_knn), and Eq. (1) is then fed the distances to the codes, which
 * is what such a search returns.  Same outputs, same limits as the calls it makes.  If some row finds fewer than k other points in its tau lists the search is
 * repeated for all rows with twice the lists, up to min(32, nlist), before TSNE_ENUM is returned;
 * *tau_used (host, may be NULL) receives the number of lists the result was built with.
 */
int tsne_build_P_approx_workspace_bytes(int32_t n, int32_t d, int32_t k, int32_t nlist, int32_t tau, int32_t pq_m,
                                        size_t *bytes);
int tsne_build_P_approx(const float *d_X, int32_t n, int32_t d, float perplexity, int32_t k, int32_t nlist,
                        int32_t tau, int32_t kmeans_iters, int32_t pq_m, int32_t *d_row_ptr, int32_t *d_col, float *d_val,
                        int64_t cap_nnz, int64_t *nnz, int32_t *d_knn_idx, float *d_knn_d2, int32_t *n_unconverged,
                        int32_t *tau_used, void *d_workspace, size_t workspace_bytes, void *stream);

/* Hands a CSR matrix P (n rows, int32 indices, float values, all on the device) to the context.
 * Borrowed: it must outlive every later call on the context (with renumbering on, the library works
 * from a relabelled private copy but still reads the original for tsne_kl).  With renumbering on,
 * nnz must not exceed max_nnz.  Column indices must lie in [0, n).  With renumbering on and
 * far_tiles = 0 or 2 the call waits for the stream (it reads back which kernel will take the far part). */
int tsne_set_P(tsne_ctx *ctx, const int32_t *d_row_ptr, const int32_t *d_col, const float *d_val, int64_t nnz);

/* How the context holds P after tsne_set_P, for byte accounting: with renumbering on, *near_entries is the
 * number of stored entries of the part near the diagonal (rows padded to multiples of 32 entries; 6 bytes each:
 * a float and a 16-bit column) and *far_entries that of the rest (8 bytes each); without renumbering
 * *near_entries = 0 and *far_entries = nnz (the caller's CSR, 8 bytes each).  Synchronises. */
int tsne_P_layout(tsne_ctx *ctx, int64_t *near_entries, int64_t *far_entries);

/* Resets the optimiser state: velocity = 0, gains = 1 (enqueued). */
int tsne_init_state(tsne_ctx *ctx);

/* Copies the optimiser state out of / into the context (device arrays of n x 2 floats);
 * with Y and the iteration index this is everything needed to stop and resume. */
int tsne_get_state(tsne_ctx *ctx, float *d_velocity, float *d_gains);
int tsne_set_state(tsne_ctx *ctx, const float *d_velocity, const float *d_gains);

/*
 * Alg. 1 lines 4-8, once: tree build over d_Y (Sec. III-C steps 1-4), repulsive forces and Z
 * (step 5, Eq. (14)-(15)), attractive forces (Eq. (5)), update with gains and momentum.
 * d_Y: n x 2 floats, interleaved, updated in place.  iter: 0-based iteration index; it selects
 * exaggeration and momentum.  Enqueues only.
 */
int tsne_step(tsne_ctx *ctx, float *d_Y, int32_t iter);

/* Alg. 1 lines 3-9: n_iter steps starting at iteration iter0; then synchronises and returns
 * TSNE_ENUM if the device reported trouble.  The result equals n_iter calls of tsne_step bit for bit.
 * Between the iterations of one call the library works from its own copy of the embedding, so d_Y is
 * read at the start, holds the final embedding on return, and is unspecified in between (and after an
 * error). */
int tsne_run(tsne_ctx *ctx, float *d_Y, int32_t iter0, int32_t n_iter);

/*
 * The forces at a fixed Y without the update (what the tests compare with the CPU oracle).
 * d_attr:  n x 2, A_i = sum_j p_ij w_ij (y_i - y_j), w = 1/(1+|y_i-y_j|^2)      (Eq. (5) times Z)
 * d_rep:   n x 2, R_i = sum over accepted cells n_c w^2 (y_i - y_c) + opened leaves (Eq. (15))
 * d_Z:     one double, the Barnes-Hut estimate of Eq. (4)
 * The gradient of Eq. (7) is 4 (alpha A - R / Z).  Any output may be NULL.  Enqueues only.
 */
int tsne_gradient(tsne_ctx *ctx, const float *d_Y, float *d_attr, float *d_rep, double *d_Z);

/*
 * Copies out the tree of the last tsne_step / tsne_gradient (device arrays, any may be NULL):
 * d_keys[n]   interleaved grid key of every point (x in even bits, 2 morton_bits bits), original order
 * d_perm[n]   spatial order: position p holds original index d_perm[p]
 * cells in depth-first pre-order, children in quadrant order, cap_cells entries each:
 * d_depth, d_lo, d_hi (member positions [lo,hi)), d_leaf (0/1), d_com (2 floats per cell)
 * d_root[3]   lower corner x, y and side of the root square
 * *n_cells (host) receives the cell count.  Synchronises.
 */
int tsne_export_tree(tsne_ctx *ctx, uint64_t *d_keys, int32_t *d_perm, int32_t cap_cells,
                     int32_t *d_depth, int32_t *d_lo, int32_t *d_hi, int32_t *d_leaf, float *d_com,
                     float *d_root, int32_t *n_cells);

/* KL(P||Q) of Sec. III-A for the embedding d_Y with the exact Z of Eq. (4) (all pairs, O(n^2)).
 * A harness utility, not part of the step.  Synchronises. */
int tsne_kl(tsne_ctx *ctx, const float *d_Y, double *kl);

/*
 * tsne_kl for callers that cannot allocate or hold a context: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same kernels and the same result as tsne_kl on the same P and Y;
 * the partial sums live in a 24 KB array inside the library's device image (one copy per GPU, kept until the
 * process ends) instead of a context's workspace.  The call allocates nothing, creates nothing and does not
 * synchronise: it enqueues four kernels on `stream`.
 * d_Y: n x 2 floats; P: CSR with n rows (d_col / d_val may be NULL only if the matrix has no entries);
 * d_out (device, caller-owned): d_out[0] = KL(P||Q), d_out[1] = the exact Z of Eq. (4).
 * n > TSNE_KL_STATIC_MAX_N returns TSNE_EINVAL (the all-pairs sum is O(n^2); beyond this size use a context).
 * All calls on one GPU share the one array: calls that overlap on the same GPU (two streams, two threads)
 * race and give wrong results; calls on one stream are ordered and safe.
 */
#define TSNE_KL_STATIC_MAX_N (1 << 22)
int tsne_kl_static(const float *d_Y, int32_t n, const int32_t *d_row_ptr, const int32_t *d_col, const float *d_val,
                   double *d_out, void *stream);

/*
 * Per-phase GPU time of tsne_step, measured with HIP events recorded on the streams the kernels
 * run on.  tsne_timing_begin() arms the next max_steps calls of tsne_step (9 events per step);
 * tsne_timing_end() synchronises, and returns the number of steps timed plus the mean milliseconds
 * per step of the four phases (any pointer may be NULL):
 *   ms[0] tree build (Sec. III-C steps 1-4)   ms[1] walk + Z (step 5)
 *   ms[2] attractive forces (Eq. (5))         ms[3] update (Alg. 1 line 8)
 * With overlap on the attractive kernel runs beside other phases, so the four do not add up
 * to the step time.
 */
int tsne_timing_begin(tsne_ctx *ctx, int32_t max_steps);
/* The same, timing only every `every`-th step (the first one included) until max_steps steps have
 * been timed: the event records cost about 30 us per timed step at N = 1.28M, which a long run
 * should not pay on every iteration. */
int tsne_timing_begin_every(tsne_ctx *ctx, int32_t max_steps, int32_t every);
int tsne_timing_end(tsne_ctx *ctx, int32_t *steps, float ms[4]);

/* Synchronises the stream and returns the device status bits (0 = fine) in *status. */
int tsne_status(tsne_ctx *ctx, uint32_t *status);

const char *tsne_strerror(int code);
const char *tsne_last_error(const tsne_ctx *ctx); /* detail of the last failure on this context */

#ifdef __cplusplus
}
#endif
#endif /* TSNE_H */
