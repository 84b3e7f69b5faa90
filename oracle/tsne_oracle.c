/*
 * tsne_oracle.c -- plain CPU reference for Barnes-Hut t-SNE (arXiv 1807.11824).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * checked against.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may load it; the product library never does and shares no
 * code, header, table or helper with it.
 *
 * Everything is written straight from the paper's definitions, in double
 * precision, with no blocking, no fusion and no intrinsics.  OpenMP is used
 * only as "parallel for" over independent points so that the timed baseline
 * uses the host's cores; it never changes the order of any floating-point sum.
 * Compile with -ffp-contract=off: the few single-precision expressions that
 * decide integers (quantisation, acceptance test) must round after every
 * operation.
 *
 * Map of the paper to the functions below
 *   Sec. III-B, Alg. 1 line 1 (K nearest neighbours, exact reading) oracle_knn
 *   Eq. (1) with sigma_i fixed by an entropy target                  oracle_cond_p
 *   p_ij = (p_i|j + p_j|i) / 2N (text after Eq. (4)), <= 2NK nnz     oracle_symmetrise
 *   Eq. (2), (4), (5), (6), (7) without approximation                oracle_grad_exact
 *   KL(P||Q), Sec. III-A                                             oracle_kl
 *   Sec. III-C steps 1, 2, 4 (bounding box, quad tree, spatial sort) oracle_morton, oracle_sort, oracle_tree
 *   Sec. III-C step 3 (cell count and centre)                        inside oracle_tree
 *   Sec. III-C step 5, Eq. (14), (15), Z estimate                    oracle_grad_bh
 *   (the ..._ties forms take a rank that orders points of equal key in step 4, which the paper
 *    leaves open; without one it is the index)
 *   Alg. 1 line 8 (apply forces)                                     oracle_update
 *   Alg. 1 lines 3-9                                                 oracle_run
 *
 * Pins (tests/test_oracle_*.py, all CPU): finite differences of KL pin
 * oracle_grad_exact; theta = 0 pins the leaf path of oracle_grad_bh to it;
 * the far-cell error bound of Eq. (15) and tree invariants pin the summary
 * path; a brute-force recursive quadtree written in Python pins oracle_tree;
 * closed forms pin Z, the two-neighbour beta and the all-equal-distance row;
 * an integer-lattice data set and scipy's k-d tree pin oracle_knn.
 * PARITY UNPINNED against anything outside the paper: the constants of
 * oracle_update (the paper prints no update rule) and the choice "radius =
 * full cell side, centre = centre of mass" in the acceptance test.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------ */
/* Sec. III-B: exact K nearest neighbours under squared Euclidean distance. */
/* Row i of the result lists the k smallest (distance, index) pairs, j != i, */
/* in lexicographic order.  Distances are accumulated over the coordinates  */
/* t = 0 .. d-1 in that order, in double.                                   */
/* rows == NULL: all n query rows; else only the n_rows rows listed.        */
/* ------------------------------------------------------------------------ */
int oracle_knn(const float *X, int32_t n, int32_t d, int32_t k,
               const int32_t *rows, int32_t n_rows,
               int32_t *idx, double *d2out)
{
    if (!X || !idx || !d2out || n < 2 || d < 1 || k < 1 || k >= n) return -1;
    int32_t nq = rows ? n_rows : n;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 4)
    for (int32_t r = 0; r < nq; ++r) {
        int32_t i = rows ? rows[r] : r;
        if (i < 0 || i >= n) { bad = 1; continue; }
        int32_t *bi = idx + (size_t)r * k;
        double *bd = d2out + (size_t)r * k;
        int32_t have = 0;
        for (int32_t j = 0; j < n; ++j) {
            if (j == i) continue;
            double s = 0.0;
            for (int32_t t = 0; t < d; ++t) {
                double diff = (double)X[(size_t)i * d + t] - (double)X[(size_t)j * d + t];
                s += diff * diff;
            }
            /* insertion into the sorted list of the best k so far; j grows, so
             * among equal distances the earlier (smaller) index stays in front */
            if (have == k && !(s < bd[k - 1])) continue;
            int32_t pos = have < k ? have : k - 1;
            while (pos > 0 && s < bd[pos - 1]) {
                bd[pos] = bd[pos - 1];
                bi[pos] = bi[pos - 1];
                --pos;
            }
            bd[pos] = s;
            bi[pos] = j;
            if (have < k) ++have;
        }
    }
    return bad ? -1 : 0;
}

/* ------------------------------------------------------------------------ */
/* Eq. (1) restricted to the k neighbours of each point.  beta = 1/(2 sigma^2) */
/* is chosen so that the Shannon entropy (natural log) of the row equals    */
/* ln(perplexity).  H(beta) is continuous and non-increasing, so: bracket   */
/* from beta = 1 by doubling / halving, then bisect.                        */
/* Returns the number of rows whose entropy could not be brought within tol */
/* (e.g. all k distances equal: H = ln k for every beta).                   */
/* ------------------------------------------------------------------------ */
static double row_entropy(const double *dd, int32_t k, double beta, double *p)
{
    /* the shift by the smallest distance cancels in Eq. (1) */
    double dmin = dd[0];
    for (int32_t m = 1; m < k; ++m) if (dd[m] < dmin) dmin = dd[m];
    double S = 0.0, T = 0.0;
    for (int32_t m = 0; m < k; ++m) {
        double e = exp(-beta * (dd[m] - dmin));
        p[m] = e;
        S += e;
        T += (dd[m] - dmin) * e;
    }
    for (int32_t m = 0; m < k; ++m) p[m] /= S;
    /* -sum p ln p with p = e/S and ln e = -beta (d - dmin) */
    return log(S) + beta * T / S;
}

int32_t oracle_cond_p(const double *d2, int32_t n_rows, int32_t k, double perplexity,
                      double tol, double *cond, double *beta_out)
{
    if (!d2 || !cond || n_rows < 1 || k < 1 || !(perplexity > 0.0)) return -1;
    const double target = log(perplexity);
    int32_t unconverged = 0;
#pragma omp parallel for schedule(static) reduction(+ : unconverged)
    for (int32_t i = 0; i < n_rows; ++i) {
        const double *dd = d2 + (size_t)i * k;
        double *p = cond + (size_t)i * k;
        double lo = 0.0, hi = INFINITY, beta = 1.0;
        int ok = 0;
        for (int it = 0; it < 400; ++it) {
            double H = row_entropy(dd, k, beta, p);
            if (fabs(H - target) <= tol) { ok = 1; break; }
            if (H > target) {            /* too flat: sharpen */
                lo = beta;
                beta = isinf(hi) ? beta * 2.0 : 0.5 * (lo + hi);
            } else {                     /* too peaked: widen */
                hi = beta;
                beta = 0.5 * (lo + hi);
            }
            if (!(beta > 0.0) || isinf(beta)) break;
        }
        if (!ok) { row_entropy(dd, k, beta, p); ++unconverged; }
        if (beta_out) beta_out[i] = beta;
    }
    return unconverged;
}

/* ------------------------------------------------------------------------ */
/* p_ij = (p_j|i + p_i|j) / (2N), absent conditionals = 0.  CSR, columns    */
/* ascending, no diagonal.  At most 2Nk entries (Sec. III-B).               */
/* Returns nnz, or -1 on bad input / too small capacity.                    */
/* ------------------------------------------------------------------------ */
typedef struct { int32_t r, c; double v; } triple_t;

static int cmp_triple(const void *a, const void *b)
{
    const triple_t *x = (const triple_t *)a, *y = (const triple_t *)b;
    if (x->r != y->r) return x->r < y->r ? -1 : 1;
    if (x->c != y->c) return x->c < y->c ? -1 : 1;
    return 0;
}

int64_t oracle_symmetrise(const int32_t *idx, const double *cond, int32_t n, int32_t k,
                          int32_t *row_ptr, int32_t *col, double *val, int64_t cap)
{
    if (!idx || !cond || !row_ptr || !col || !val || n < 1 || k < 1) return -1;
    size_t m = (size_t)n * k;
    triple_t *t = (triple_t *)malloc(2 * m * sizeof(triple_t));
    if (!t) return -1;
    for (int32_t i = 0; i < n; ++i)
        for (int32_t a = 0; a < k; ++a) {
            int32_t j = idx[(size_t)i * k + a];
            double v = cond[(size_t)i * k + a];
            if (j < 0 || j >= n || j == i) { free(t); return -1; }
            size_t e = 2 * ((size_t)i * k + a);
            t[e].r = i; t[e].c = j; t[e].v = v;           /* p_j|i at (i,j) */
            t[e + 1].r = j; t[e + 1].c = i; t[e + 1].v = v; /* and at (j,i)  */
        }
    qsort(t, 2 * m, sizeof(triple_t), cmp_triple);
    int64_t nnz = 0;
    memset(row_ptr, 0, ((size_t)n + 1) * sizeof(int32_t));
    size_t e = 0;
    while (e < 2 * m) {
        size_t f = e + 1;
        double s = t[e].v;
        while (f < 2 * m && t[f].r == t[e].r && t[f].c == t[e].c) { s += t[f].v; ++f; }
        if (f - e > 2 || nnz >= cap) { free(t); return -1; } /* duplicate neighbour in a row */
        col[nnz] = t[e].c;
        val[nnz] = s / (2.0 * (double)n);
        row_ptr[t[e].r + 1] += 1;
        ++nnz;
        e = f;
    }
    for (int32_t i = 0; i < n; ++i) row_ptr[i + 1] += row_ptr[i];
    free(t);
    return nnz;
}

/* ------------------------------------------------------------------------ */
/* Exact gradient.  w_ij = 1/(1+|y_i-y_j|^2) (numerator of Eq. (2));        */
/* Z = sum over ordered pairs k != l of w_kl (Eq. (4));                     */
/* A_i = sum_j p_ij w_ij (y_i-y_j)           = F_attr of Eq. (5), q Z = w;  */
/* R_i = sum_{j != i} w_ij^2 (y_i-y_j)       = -Z F_rep of Eq. (6);         */
/* grad_i = 4 (alpha A_i - R_i / Z)          Eq. (7), alpha = exaggeration. */
/* Y: n x 2 doubles.  P in CSR with double values.                          */
/* ------------------------------------------------------------------------ */
void oracle_grad_exact(const double *Y, int32_t n, const int32_t *row_ptr, const int32_t *col,
                       const double *val, double alpha,
                       double *A, double *R, double *Zout, double *grad)
{
    double Z = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : Z)
    for (int32_t i = 0; i < n; ++i) {
        double rx = 0.0, ry = 0.0, z = 0.0;
        for (int32_t j = 0; j < n; ++j) {
            if (j == i) continue;
            double dx = Y[2 * i] - Y[2 * j], dy = Y[2 * i + 1] - Y[2 * j + 1];
            double w = 1.0 / (1.0 + dx * dx + dy * dy);
            z += w;
            rx += w * w * dx;
            ry += w * w * dy;
        }
        R[2 * i] = rx; R[2 * i + 1] = ry;
        Z += z;
        double ax = 0.0, ay = 0.0;
        for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            int32_t j = col[e];
            double dx = Y[2 * i] - Y[2 * j], dy = Y[2 * i + 1] - Y[2 * j + 1];
            double w = 1.0 / (1.0 + dx * dx + dy * dy);
            ax += val[e] * w * dx;
            ay += val[e] * w * dy;
        }
        A[2 * i] = ax; A[2 * i + 1] = ay;
    }
    if (Zout) *Zout = Z;
    if (grad)
        for (int32_t i = 0; i < 2 * n; ++i) grad[i] = 4.0 * (alpha * A[i] - R[i] / Z);
}

/* Attractive term alone (Eq. (5)), used when timing the Barnes-Hut step.   */
void oracle_attract(const double *Y, int32_t n, const int32_t *row_ptr, const int32_t *col,
                    const double *val, double *A)
{
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < n; ++i) {
        double ax = 0.0, ay = 0.0;
        for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            int32_t j = col[e];
            double dx = Y[2 * i] - Y[2 * j], dy = Y[2 * i + 1] - Y[2 * j + 1];
            double w = 1.0 / (1.0 + dx * dx + dy * dy);
            ax += val[e] * w * dx;
            ay += val[e] * w * dy;
        }
        A[2 * i] = ax; A[2 * i + 1] = ay;
    }
}

/* KL(P||Q) = sum_ij p_ij ln(p_ij / q_ij), q_ij = w_ij / Z (Eq. (2), (4)),  */
/* summed over the stored entries of P (0 ln 0 = 0).  Exact Z, O(N^2).      */
double oracle_kl(const double *Y, int32_t n, const int32_t *row_ptr, const int32_t *col,
                 const double *val)
{
    double Z = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : Z)
    for (int32_t i = 0; i < n; ++i) {
        double z = 0.0;
        for (int32_t j = 0; j < n; ++j) {
            if (j == i) continue;
            double dx = Y[2 * i] - Y[2 * j], dy = Y[2 * i + 1] - Y[2 * j + 1];
            z += 1.0 / (1.0 + dx * dx + dy * dy);
        }
        Z += z;
    }
    double kl = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : kl)
    for (int32_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            int32_t j = col[e];
            if (!(val[e] > 0.0)) continue;
            double dx = Y[2 * i] - Y[2 * j], dy = Y[2 * i + 1] - Y[2 * j + 1];
            double q = 1.0 / ((1.0 + dx * dx + dy * dy) * Z);
            s += val[e] * log(val[e] / q);
        }
        kl += s;
    }
    return kl;
}

/* ------------------------------------------------------------------------ */
/* Sec. III-C step 1 and the quantisation that places points in the quad    */
/* tree.  Root square: lower corner (min x, min y), side W = smallest power */
/* of two >= max(extent x, extent y), never below 2^-40.  Each coordinate   */
/* is quantised to `bits` bits in SINGLE precision, one rounding per        */
/* operation; the key interleaves x into the even and y into the odd bits.  */
/* bits <= 24: a float has 24 significant bits, a finer grid cannot tell    */
/* two different coordinates apart any better.                              */
/* root[0..2] = x0, y0, W.  Returns -1 if a coordinate is not finite.       */
/* ------------------------------------------------------------------------ */
int oracle_morton(const float *Y, int32_t n, int32_t bits, float *root, uint64_t *keys)
{
    if (!Y || !root || !keys || n < 1 || bits < 1 || bits > 24) return -1;
    float minx = Y[0], maxx = Y[0], miny = Y[1], maxy = Y[1];
    for (int32_t i = 0; i < n; ++i) {
        float x = Y[2 * i], y = Y[2 * i + 1];
        if (!isfinite(x) || !isfinite(y)) return -1;
        if (x < minx) minx = x;
        if (x > maxx) maxx = x;
        if (y < miny) miny = y;
        if (y > maxy) maxy = y;
    }
    volatile float ex = maxx - minx, ey = maxy - miny;
    float e = ex > ey ? ex : ey;
    float W = ldexpf(1.0f, -40);
    while (W < e) W *= 2.0f;
    volatile float S = ldexpf(1.0f, bits) / W;      /* exact: power of two */
    uint32_t qmax = (1u << bits) - 1u;
    root[0] = minx; root[1] = miny; root[2] = W;
    for (int32_t i = 0; i < n; ++i) {
        volatile float rx = Y[2 * i] - minx, ry = Y[2 * i + 1] - miny;
        volatile float sx = rx * S, sy = ry * S;
        float fx = floorf(sx), fy = floorf(sy);
        uint32_t qx = fx >= (float)qmax ? qmax : (uint32_t)fx;
        uint32_t qy = fy >= (float)qmax ? qmax : (uint32_t)fy;
        uint64_t key = 0;
        for (int32_t b = 0; b < bits; ++b) {
            key |= (uint64_t)((qx >> b) & 1u) << (2 * b);
            key |= (uint64_t)((qy >> b) & 1u) << (2 * b + 1);
        }
        keys[i] = key;
    }
    return 0;
}

/* Sec. III-C step 4: order points along the curve.  The paper leaves the    */
/* order of points with equal keys open; the reading here is: by original    */
/* index.  tie_rank (may be NULL) replaces the index in that role: a test    */
/* that checks an implementation which orders equal keys otherwise passes    */
/* the rank it found there, after checking that the order is a sorted one.   */
typedef struct { uint64_t key; int32_t tie, idx; } keyidx_t;

static int cmp_keyidx(const void *a, const void *b)
{
    const keyidx_t *x = (const keyidx_t *)a, *y = (const keyidx_t *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->tie != y->tie) return x->tie < y->tie ? -1 : 1;
    if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1;
    return 0;
}

int oracle_sort_ties(const uint64_t *keys, int32_t n, const int32_t *tie_rank, uint64_t *sorted_keys, int32_t *perm)
{
    keyidx_t *t = (keyidx_t *)malloc((size_t)n * sizeof(keyidx_t));
    if (!t) return -1;
    for (int32_t i = 0; i < n; ++i) { t[i].key = keys[i]; t[i].tie = tie_rank ? tie_rank[i] : i; t[i].idx = i; }
    qsort(t, (size_t)n, sizeof(keyidx_t), cmp_keyidx);
    for (int32_t i = 0; i < n; ++i) { sorted_keys[i] = t[i].key; perm[i] = t[i].idx; }
    free(t);
    return 0;
}

int oracle_sort(const uint64_t *keys, int32_t n, uint64_t *sorted_keys, int32_t *perm)
{
    return oracle_sort_ties(keys, n, NULL, sorted_keys, perm);
}

/* ------------------------------------------------------------------------ */
/* Sec. III-C steps 2 and 3.  The quad tree over the sorted keys: the root  */
/* covers [0,n) at depth 0; a cell at depth t is a leaf when it holds at    */
/* most leaf_cap points or t == bits, otherwise it has one child per        */
/* non-empty quadrant (the next two key bits), which is a contiguous        */
/* sub-range.  Cells are emitted in depth-first pre-order, children in      */
/* quadrant order.  For every cell: count = hi - lo and centre of mass =    */
/* mean of its points (summed in double in sorted order, rounded to float). */
/* ------------------------------------------------------------------------ */
typedef struct {
    const uint64_t *keys;   /* sorted */
    const float *Ys;        /* points in sorted order, n x 2 */
    int32_t bits, leaf_cap, cap, m;
    int32_t *depth, *lo, *hi, *leaf, *child; /* child: 4 per node, -1 = none */
    uint64_t *prefix;
    float *com;             /* 2 per node */
    int overflow;
} treeb_t;

static int32_t tree_rec(treeb_t *T, int32_t lo, int32_t hi, int32_t depth, uint64_t prefix)
{
    if (T->m >= T->cap) { T->overflow = 1; return -1; }
    int32_t id = T->m++;
    T->depth[id] = depth; T->lo[id] = lo; T->hi[id] = hi; T->prefix[id] = prefix;
    double sx = 0.0, sy = 0.0;
    for (int32_t p = lo; p < hi; ++p) { sx += (double)T->Ys[2 * p]; sy += (double)T->Ys[2 * p + 1]; }
    T->com[2 * id] = (float)(sx / (double)(hi - lo));
    T->com[2 * id + 1] = (float)(sy / (double)(hi - lo));
    for (int q = 0; q < 4; ++q) T->child[4 * id + q] = -1;
    int is_leaf = (hi - lo <= T->leaf_cap) || depth == T->bits;
    T->leaf[id] = is_leaf;
    if (is_leaf) return id;
    int shift = 2 * (T->bits - depth - 1);
    int32_t p = lo;
    for (uint64_t q = 0; q < 4; ++q) {
        int32_t s = p;
        while (p < hi && ((T->keys[p] >> shift) & 3u) == q) ++p;
        if (p > s) T->child[4 * id + q] = tree_rec(T, s, p, depth + 1, (prefix << 2) | q);
    }
    return id;
}

int32_t oracle_tree(const uint64_t *sorted_keys, const float *Ys, int32_t n, int32_t bits,
                    int32_t leaf_cap, int32_t cap,
                    int32_t *depth, uint64_t *prefix, int32_t *lo, int32_t *hi, int32_t *leaf,
                    int32_t *child, float *com)
{
    if (n < 1 || bits < 1 || bits > 24 || leaf_cap < 1) return -1;
    treeb_t T = { sorted_keys, Ys, bits, leaf_cap, cap, 0, depth, lo, hi, leaf, child, prefix, com, 0 };
    tree_rec(&T, 0, n, 0, 0u);
    return T.overflow ? -1 : T.m;
}

/* ------------------------------------------------------------------------ */
/* Sec. III-C step 5: repulsive forces by depth-first search with the       */
/* acceptance test of Eq. (14) and the cell summary of Eq. (15); the same   */
/* walk accumulates the estimate of Z (last paragraph before the 5 steps).  */
/*                                                                          */
/* Points are handled in groups of `group` consecutive positions of the     */
/* sorted order (group = 1 is the per-point search of the text; a larger    */
/* group makes all its points take the same decisions, which is how a tree  */
/* code keeps the lanes of one wavefront together).  A cell is accepted for */
/* a group when Eq. (14) holds for EVERY point of the group, with r_cell =  */
/* side of the cell and y_cell = its centre of mass.  The test is evaluated */
/* in single precision, squared, one rounding per operation (the sum of the */
/* two squares is one fused multiply-add):                                  */
/*      side^2 < theta^2 * ((y_i - y_cell).y^2 + (y_i - y_cell).x^2).       */
/* Accepted cell: every point of the group gets n w^2 (y_i - y_cell) and    */
/* n w, w = 1/(1+|y_i - y_cell|^2).  Rejected inner cell: descend into its  */
/* children.  Rejected leaf: its points are taken one by one, j = i skipped */
/* by index.                                                                */
/* Outputs are indexed by ORIGINAL point index: R (n x 2), z (n).           */
/* stats[0..2] += accepted cells, opened leaves, point-point terms (per     */
/* group, i.e. not multiplied by the group size).                           */
/* ------------------------------------------------------------------------ */
typedef struct {
    const treeb_t *T;
    const float *Ys;
    float W, theta2;
    int32_t g0, g1;          /* positions of the group */
    double *rx, *ry, *z;     /* per member of the group */
    int64_t st[3];
} walk_t;

static void walk_rec(walk_t *K, int32_t id)
{
    const treeb_t *T = K->T;
    volatile float side = ldexpf(K->W, -T->depth[id]);
    volatile float side2 = side * side;
    float cx = T->com[2 * id], cy = T->com[2 * id + 1];
    int all_pass = 1;
    for (int32_t p = K->g0; p < K->g1 && all_pass; ++p) {
        volatile float dx = K->Ys[2 * p] - cx, dy = K->Ys[2 * p + 1] - cy;
        volatile float dx2 = dx * dx;
        volatile float dist2 = fmaf(dy, dy, dx2);
        volatile float rhs = K->theta2 * dist2;
        if (!(side2 < rhs)) all_pass = 0;
    }
    if (all_pass) {
        double n = (double)(T->hi[id] - T->lo[id]);
        for (int32_t p = K->g0; p < K->g1; ++p) {
            double ddx = (double)K->Ys[2 * p] - (double)cx, ddy = (double)K->Ys[2 * p + 1] - (double)cy;
            double w = 1.0 / (1.0 + ddx * ddx + ddy * ddy);
            K->z[p - K->g0] += n * w;
            K->rx[p - K->g0] += n * w * w * ddx;
            K->ry[p - K->g0] += n * w * w * ddy;
        }
        K->st[0] += 1;
        return;
    }
    if (!T->leaf[id]) {
        for (int q = 0; q < 4; ++q)
            if (T->child[4 * id + q] >= 0) walk_rec(K, T->child[4 * id + q]);
        return;
    }
    K->st[1] += 1;
    K->st[2] += T->hi[id] - T->lo[id];
    for (int32_t p = K->g0; p < K->g1; ++p)
        for (int32_t j = T->lo[id]; j < T->hi[id]; ++j) {
            if (j == p) continue;
            double ddx = (double)K->Ys[2 * p] - (double)K->Ys[2 * j];
            double ddy = (double)K->Ys[2 * p + 1] - (double)K->Ys[2 * j + 1];
            double w = 1.0 / (1.0 + ddx * ddx + ddy * ddy);
            K->z[p - K->g0] += w;
            K->rx[p - K->g0] += w * w * ddx;
            K->ry[p - K->g0] += w * w * ddy;
        }
}

/* Whole repulsive side at fixed Y (single precision in, widened).          */
/* Returns the number of tree cells, or -1.                                 */
int32_t oracle_repulse_bh_ties(const float *Y, int32_t n, float theta, int32_t leaf_cap, int32_t group,
                               int32_t bits, const int32_t *tie_rank, double *R, double *z, double *Zout,
                               int64_t *stats)
{
    if (!Y || n < 1 || group < 1 || !(theta >= 0.0f)) return -1;
    /* leaves are disjoint and non-empty (at most n of them); an inner cell holds more than
     * leaf_cap points, so every level above the deepest has at most n / (leaf_cap + 1) */
    if (leaf_cap < 1 || bits < 1) return -1;
    int64_t cap64 = (int64_t)n + (int64_t)bits * (n / ((int64_t)leaf_cap + 1)) + 1;
    if (cap64 > 0x7FFFFFFF) return -1;
    int32_t cap = (int32_t)cap64;
    uint64_t *keys = malloc((size_t)n * 8), *skeys = malloc((size_t)n * 8);
    int32_t *perm = malloc((size_t)n * 4);
    float *Ys = malloc((size_t)n * 8);
    int32_t *depth = malloc((size_t)cap * 4), *lo = malloc((size_t)cap * 4), *hi = malloc((size_t)cap * 4);
    int32_t *leaf = malloc((size_t)cap * 4), *child = malloc((size_t)cap * 16);
    uint64_t *prefix = malloc((size_t)cap * 8);
    float *com = malloc((size_t)cap * 8);
    float root[3];
    int32_t m = -1;
    if (keys && skeys && perm && Ys && depth && lo && hi && leaf && child && prefix && com &&
        oracle_morton(Y, n, bits, root, keys) == 0 && oracle_sort_ties(keys, n, tie_rank, skeys, perm) == 0) {
        for (int32_t p = 0; p < n; ++p) { Ys[2 * p] = Y[2 * perm[p]]; Ys[2 * p + 1] = Y[2 * perm[p] + 1]; }
        m = oracle_tree(skeys, Ys, n, bits, leaf_cap, cap, depth, prefix, lo, hi, leaf, child, com);
    }
    if (m > 0) {
        treeb_t T = { skeys, Ys, bits, leaf_cap, cap, m, depth, lo, hi, leaf, child, prefix, com, 0 };
        volatile float th2 = theta * theta;
        int32_t n_groups = (n + group - 1) / group;
        double Z = 0.0;
        int64_t s0 = 0, s1 = 0, s2 = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : Z, s0, s1, s2)
        for (int32_t g = 0; g < n_groups; ++g) {
            walk_t K;
            K.T = &T; K.Ys = Ys; K.W = root[2]; K.theta2 = th2;
            K.g0 = g * group; K.g1 = K.g0 + group < n ? K.g0 + group : n;
            int32_t gs = K.g1 - K.g0;
            K.rx = calloc((size_t)gs, 8); K.ry = calloc((size_t)gs, 8); K.z = calloc((size_t)gs, 8);
            K.st[0] = K.st[1] = K.st[2] = 0;
            walk_rec(&K, 0);
            for (int32_t p = K.g0; p < K.g1; ++p) {
                int32_t i = perm[p];
                R[2 * i] = K.rx[p - K.g0]; R[2 * i + 1] = K.ry[p - K.g0];
                if (z) z[i] = K.z[p - K.g0];
                Z += K.z[p - K.g0];
            }
            s0 += K.st[0]; s1 += K.st[1]; s2 += K.st[2];
            free(K.rx); free(K.ry); free(K.z);
        }
        if (Zout) *Zout = Z;
        if (stats) { stats[0] = s0; stats[1] = s1; stats[2] = s2; }
    }
    free(keys); free(skeys); free(perm); free(Ys); free(depth); free(lo); free(hi);
    free(leaf); free(child); free(prefix); free(com);
    return m;
}

int32_t oracle_repulse_bh(const float *Y, int32_t n, float theta, int32_t leaf_cap, int32_t group,
                          int32_t bits, double *R, double *z, double *Zout, int64_t *stats)
{
    return oracle_repulse_bh_ties(Y, n, theta, leaf_cap, group, bits, NULL, R, z, Zout, stats);
}

/* Barnes-Hut gradient at fixed Y: Eq. (7) with the attractive term summed  */
/* over the stored entries of P and the repulsive term / Z from the walk.   */
int32_t oracle_grad_bh_ties(const float *Y, int32_t n, const int32_t *row_ptr, const int32_t *col,
                            const double *val, float theta, int32_t leaf_cap, int32_t group, int32_t bits,
                            const int32_t *tie_rank, double alpha, double *A, double *R, double *Zout,
                            double *grad, int64_t *stats)
{
    double *Yd = malloc((size_t)n * 16);
    if (!Yd) return -1;
    for (int32_t i = 0; i < 2 * n; ++i) Yd[i] = (double)Y[i];
    oracle_attract(Yd, n, row_ptr, col, val, A);
    free(Yd);
    double Z = 0.0;
    int32_t m = oracle_repulse_bh_ties(Y, n, theta, leaf_cap, group, bits, tie_rank, R, NULL, &Z, stats);
    if (m < 0) return m;
    if (Zout) *Zout = Z;
    if (grad)
        for (int32_t i = 0; i < 2 * n; ++i) grad[i] = 4.0 * (alpha * A[i] - R[i] / Z);
    return m;
}

int32_t oracle_grad_bh(const float *Y, int32_t n, const int32_t *row_ptr, const int32_t *col,
                       const double *val, float theta, int32_t leaf_cap, int32_t group, int32_t bits,
                       double alpha, double *A, double *R, double *Zout, double *grad, int64_t *stats)
{
    return oracle_grad_bh_ties(Y, n, row_ptr, col, val, theta, leaf_cap, group, bits, NULL, alpha, A, R, Zout, grad,
                               stats);
}

/* ------------------------------------------------------------------------ */
/* Alg. 1 line 8.  The paper names the step but prints no rule; this is the */
/* customary t-SNE rule: per coordinate, the gain grows by gain_inc when    */
/* gradient and velocity disagree in sign (sign is -1, 0 or +1, so the rule */
/* is the same for a configuration and its mirror image) and shrinks by the */
/* factor gain_dec otherwise, is floored at gain_min; velocity = momentum * */
/* velocity - lr * gain * grad; Y += velocity.                              */
/* ------------------------------------------------------------------------ */
static int sign3(double x) { return x > 0.0 ? 1 : (x < 0.0 ? -1 : 0); }

void oracle_update(double *Y, double *uY, double *gains, const double *grad, int32_t n,
                   double momentum, double lr, double gain_inc, double gain_dec, double gain_min)
{
    for (int32_t c = 0; c < 2 * n; ++c) {
        double g = gains[c];
        if (sign3(grad[c]) != sign3(uY[c])) g = g + gain_inc; else g = g * gain_dec;
        if (g < gain_min) g = gain_min;
        gains[c] = g;
        uY[c] = momentum * uY[c] - lr * g * grad[c];
        Y[c] += uY[c];
    }
}

/* Alg. 1 lines 3-9 for n_iter iterations starting at iteration `iter0`.    */
/* State (Y, uY, gains) is double; the tree of each iteration is built from */
/* Y rounded to single precision, as the library's is.                      */
typedef struct {
    float theta; int32_t leaf_cap, group, bits;
    double lr, exaggeration; int32_t exaggeration_iters;
    double momentum_early, momentum_late; int32_t momentum_switch_iter;
    double gain_inc, gain_dec, gain_min;
} oracle_run_params;

int oracle_run(double *Y, double *uY, double *gains, int32_t n, const int32_t *row_ptr,
               const int32_t *col, const double *val, const oracle_run_params *pr,
               int32_t iter0, int32_t n_iter)
{
    float *Yf = malloc((size_t)n * 8);
    double *A = malloc((size_t)n * 16), *R = malloc((size_t)n * 16), *grad = malloc((size_t)n * 16);
    int rc = 0;
    if (!Yf || !A || !R || !grad) rc = -1;
    for (int32_t it = iter0; rc == 0 && it < iter0 + n_iter; ++it) {
        double alpha = it < pr->exaggeration_iters ? pr->exaggeration : 1.0;
        double mom = it < pr->momentum_switch_iter ? pr->momentum_early : pr->momentum_late;
        for (int32_t c = 0; c < 2 * n; ++c) Yf[c] = (float)Y[c];
        double Z;
        if (pr->theta > 0.0f) {
            /* attraction from the double state; the tree and the walk from its rounding */
            oracle_attract(Y, n, row_ptr, col, val, A);
            if (oracle_repulse_bh(Yf, n, pr->theta, pr->leaf_cap, pr->group, pr->bits, R, NULL, &Z, NULL) < 0) rc = -1;
            for (int32_t c = 0; c < 2 * n; ++c) grad[c] = 4.0 * (alpha * A[c] - R[c] / Z);
        } else {
            oracle_grad_exact(Y, n, row_ptr, col, val, alpha, A, R, &Z, grad);
        }
        if (rc == 0)
            oracle_update(Y, uY, gains, grad, n, mom, pr->lr, pr->gain_inc, pr->gain_dec, pr->gain_min);
    }
    free(Yf); free(A); free(R); free(grad);
    return rc;
}

int32_t oracle_threads(void)
{
    int32_t t = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        t = (int32_t)omp_get_num_threads();
    }
#endif
    return t;
}
