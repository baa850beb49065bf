/*
 * CPU oracle for the kernel matrix-vector product y = K(X,X) b and for the
 * F3M approximation of it (arXiv 2202.01085); the last section does the same for
 * two point sets, v = K(X,Y) b (readings R8-R11 there).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 statement of
 * what the GPU library has to compute; nothing in the product path may call
 * it.  It shares no code, header, table or constant with the HIP sources.
 *
 * What follows the paper, and where:
 *   - exact product v_i = sum_j k(x_i,y_j) b_j ............ Sec. 2 (KeOps paragraph)
 *   - Gaussian kernel exp(-|x-y|^2/(2 gamma^2)) ........... Sec. 5, first paragraph
 *   - enclosing cube edge E, anchored at the per-dim min .. Sec. 3 "Enclosing and
 *                                                            partitioning the data",
 *                                                            Sec. 4.2 box-index formula
 *   - box index of a point at a depth ..................... Sec. 4.2 box-index formula
 *   - empty boxes are dropped ............................. Sec. 4.2 "Removing empty boxes"
 *   - far iff |centre_x - centre_y| >= 2 l, l = E/2^depth . Sec. 3 "Far and near-field"
 *   - new pairs = children x children of old near pairs ... Sec. 4.1 "Ensuring
 *                                                            interactions are sorted"
 *   - Chebyshev nodes of the 2nd kind, Lagrange basis ..... Sec. 3 "Lagrange interpolation"
 *   - barycentric form and its weights .................... Appendix C
 *   - v ~ L_X^T (K (L_Y b)) for a far pair ................ Sec. 3 "Interpolating k(x,y)"
 *   - driver loop, stop on the MAXIMUM box size ........... Appendix E, Algorithm 1
 *
 * Readings where the paper is silent or garbled (each is listed in the
 * design document of the repository as well):
 *   R1  interp_nodes p = nodes PER DIMENSION, s_i = cos(i pi/(p-1)), i=0..p-1;
 *       the grid of a box has r = p^D nodes; flat node index i = sum_d i_d p^d.
 *   R2  the cell of a point is fixed ONCE, in fp32, at the quantisation depth
 *       Lq(D):  c_d = min( trunc( fl32( fl32(x_d - alpha_d) * s ) ), 2^Lq - 1 ),
 *       s = fl32( 2^Lq / E ), E = max_d fl32(max_d - min_d); the cell at depth
 *       l <= Lq is c_d >> (Lq - l).  This is the floor formula of Sec. 4.2 with
 *       its rounding spelled out; the clamp covers the points on the max face.
 *       Everything else in this file is fp64.
 *   R3  a box is identified by its integer cell vector; boxes are ordered by
 *       the bit-interleaved key (bit k of c_d -> key bit k*D + d), points inside
 *       the finest cell by original index.  The row-major index beta of
 *       Sec. 4.2 is also available (oracle_beta) and must induce the same
 *       partition.
 *   R4  far iff sum_d o_d^2 >= theta^2 with o the integer cell offset: this is
 *       |delta centre| >= theta*l divided by l, free of rounding.  theta = 2 in
 *       the paper.
 *   R5  ordered pairs (target p, source q); (p,p) is always near; the j = i
 *       term is part of the sum.
 *   R6  depth L = first depth whose largest box has <= zeta points, capped by
 *       max_depth and Lq; if E == 0 (all points equal) L = 0.
 *   R7  centre of cell c at depth l: alpha + (c + 1/2) * E/2^l; local
 *       coordinate t = (x - centre) / (l/2).
 *
 * PINS (tests/test_oracle_*.py, none needs a GPU): hand-expanded tiny sums,
 * closed forms of nodes and barycentric weights, partition of unity and
 * monomial reproduction, charge conservation of P2M, exactness of the whole
 * far-field machinery for kernels that are polynomials of degree < p per
 * coordinate, all-near == brute force, symmetry of the F3M operator, pair
 * coverage = n^2, interior neighbour counts 27/189 in 3-D, recursive lists ==
 * brute-force all-pairs classification, error falling with p.
 * Unpinned by the paper: the value of zeta and the ordering conventions (R3).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MAX_D 7
#define ORACLE_MAX_LEVELS 24

/* ------------------------------------------------------------------ */
/* kernels                                                              */
/* ------------------------------------------------------------------ */
/* kernel_id 0: Gaussian exp(-|x-y|^2 / (2 gamma^2))        (the paper's)
 * kernel_id 1: constant 1                                  (test only)
 * kernel_id 2: prod_d sum_{k=0..kparam} (x_d y_d)^k        (test only; a
 *              polynomial of degree kparam in every coordinate)          */
static double kernel_eval(int kernel_id, int kparam, double gamma, int D,
                          const double *x, const double *y)
{
    if (kernel_id == 0) {
        double r2 = 0.0;
        for (int d = 0; d < D; ++d) {
            double diff = x[d] - y[d];
            r2 += diff * diff;
        }
        return exp(-r2 / (2.0 * gamma * gamma));
    }
    if (kernel_id == 1)
        return 1.0;
    double prod = 1.0;
    for (int d = 0; d < D; ++d) {
        double z = x[d] * y[d], term = 1.0, sum = 1.0;
        for (int k = 1; k <= kparam; ++k) {
            term *= z;
            sum += term;
        }
        prod *= sum;
    }
    return prod;
}

/* Progress lines on stderr, one per finished step of a tree build or a product (for runs on
 * inputs of 1e8 .. 1e9 points that take minutes); off by default. */
static int g_verbose = 0;
void oracle_set_verbose(int on) { g_verbose = on; }
#define PROGRESS(...) do { if (g_verbose) { fprintf(stderr, "[oracle] " __VA_ARGS__); fputc('\n', stderr); fflush(stderr); } } while (0)

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* exact product                                                        */
/* ------------------------------------------------------------------ */
/* y_i = sum_{j=0..n-1} k(x_i, x_j) b_j for the rows listed in rows[0..m)
 * (rows == NULL: all rows, m == n).  X is n x D row-major fp32, widened to
 * double before any arithmetic. */
void oracle_rows_k(const float *X, int64_t n, int D, double gamma,
                   int kernel_id, int kparam, const float *b,
                   const int64_t *rows, int64_t m, double *y)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t a = 0; a < m; ++a) {
        int64_t i = rows ? rows[a] : a;
        double xi[ORACLE_MAX_D], xj[ORACLE_MAX_D];
        for (int d = 0; d < D; ++d)
            xi[d] = (double)X[i * D + d];
        double acc = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            for (int d = 0; d < D; ++d)
                xj[d] = (double)X[j * D + d];
            acc += kernel_eval(kernel_id, kparam, gamma, D, xi, xj) * (double)b[j];
        }
        y[a] = acc;
    }
}

void oracle_direct(const float *X, int64_t n, int D, double gamma,
                   const float *b, double *y)
{
    oracle_rows_k(X, n, D, gamma, 0, 0, b, NULL, n, y);
}

void oracle_rows(const float *X, int64_t n, int D, double gamma,
                 const float *b, const int64_t *rows, int64_t m, double *y)
{
    oracle_rows_k(X, n, D, gamma, 0, 0, b, rows, m, y);
}

/* ------------------------------------------------------------------ */
/* interpolation                                                        */
/* ------------------------------------------------------------------ */
/* Chebyshev nodes of the second kind, p of them: s_i = cos(i pi/(p-1)). */
void oracle_cheb2_nodes(int p, double *s)
{
    for (int i = 0; i < p; ++i)
        s[i] = cos((double)i * M_PI / (double)(p - 1));
}

/* Product form: L_i(t) = prod_{j != i} (t - s_j)/(s_i - s_j). */
void oracle_lagrange_product(int p, const double *s, double t, double *L)
{
    for (int i = 0; i < p; ++i) {
        double num = 1.0, den = 1.0;
        for (int j = 0; j < p; ++j) {
            if (j == i)
                continue;
            num *= t - s[j];
            den *= s[i] - s[j];
        }
        L[i] = num / den;
    }
}

/* Barycentric form with the closed-form weights w_i = (-1)^i delta_i,
 * delta = 1/2 at both ends; L_i(s_j) = delta_ij when t hits a node. */
void oracle_lagrange_barycentric(int p, const double *s, double t, double *L)
{
    for (int j = 0; j < p; ++j) {
        if (t == s[j]) {
            for (int i = 0; i < p; ++i)
                L[i] = (i == j) ? 1.0 : 0.0;
            return;
        }
    }
    double sum = 0.0;
    for (int i = 0; i < p; ++i) {
        double w = ((i % 2) ? -1.0 : 1.0) * ((i == 0 || i == p - 1) ? 0.5 : 1.0);
        L[i] = w / (t - s[i]);
        sum += L[i];
    }
    for (int i = 0; i < p; ++i)
        L[i] /= sum;
}

/* ------------------------------------------------------------------ */
/* tree                                                                 */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t nb;        /* occupied boxes at this depth                   */
    uint64_t *key;     /* [nb] interleaved key of the box, ascending     */
    int64_t *start;    /* [nb+1] index interval into the permuted points */
    int64_t *parent;   /* [nb] rank of the parent box one depth up       */
    int64_t *cstart;   /* [nb+1] rank interval of the children one depth down (filled when divided) */
    int64_t *near_ptr, *near_col; /* CSR by target rank, columns ascending */
    int64_t *far_ptr, *far_col;
    int64_t *small_ptr, *small_col; /* small-field pairs (Sec. 4.2): computed directly at this depth */
} olevel;

typedef struct {
    int64_t n;
    int D, Lq, L;
    double alpha[ORACLE_MAX_D];
    double E;
    float s_f;
    uint32_t *cell;    /* [n*D] cells at depth Lq, ORIGINAL point order */
    uint64_t *pkey;    /* [n] key at depth Lq, PERMUTED order            */
    int64_t *perm;     /* [n] perm[k] = original index of the k-th point in box order */
    olevel lev[ORACLE_MAX_LEVELS + 1];
    /* smooth field (Sec. 4.3): depth at which every adjacent pair is interpolated, or -1 */
    int smooth_depth;
    double gamma;      /* lengthscale the smooth rule was evaluated with (0: rule off) */
    uint8_t *rows_mark; /* NULL, or [n] in box order: 1 for the points of the row subset whose boxes have
                          interaction rows (oracle_tree_build_rows); every other row of the lists is empty */
} otree;

/* quantisation depth: as deep as a 32-bit key allows, at most 20 */
int oracle_quant_depth(int D)
{
    int q = 32 / D;
    return q > 20 ? 20 : q;
}

static uint64_t interleave(const uint32_t *c, int D, int depth)
{
    uint64_t key = 0;
    for (int k = 0; k < depth; ++k)
        for (int d = 0; d < D; ++d)
            key |= (uint64_t)((c[d] >> k) & 1u) << (k * D + d);
    return key;
}

static void deinterleave(uint64_t key, int D, int depth, int64_t *c)
{
    for (int d = 0; d < D; ++d)
        c[d] = 0;
    for (int k = 0; k < depth; ++k)
        for (int d = 0; d < D; ++d)
            c[d] |= (int64_t)((key >> (k * D + d)) & 1u) << k;
}

typedef struct {
    uint64_t key;
    int64_t idx;
} keyidx;

static int cmp_keyidx(const void *a, const void *b)
{
    const keyidx *p = (const keyidx *)a, *q = (const keyidx *)b;
    if (p->key != q->key)
        return p->key < q->key ? -1 : 1;
    return p->idx < q->idx ? -1 : (p->idx > q->idx);
}

/* Ascending (key, index).  All pairs are distinct, so the result is unique: qsort for
 * small inputs; for large ones the pairs are first dealt into 4096 buckets by the top bits
 * of the key (buckets ascend with the key) and every bucket is handed to qsort, the
 * buckets in parallel.  Same order either way. */
static void sort_keyidx(keyidx *ki, int64_t n, int key_bits)
{
    enum { BUCKET_BITS = 12, NBUCKET = 1 << BUCKET_BITS };
    if (n < ((int64_t)1 << 20) || key_bits <= BUCKET_BITS) {
        qsort(ki, (size_t)n, sizeof(keyidx), cmp_keyidx);
        return;
    }
    int shift = key_bits - BUCKET_BITS;
    int64_t *first = (int64_t *)calloc((size_t)NBUCKET + 1, sizeof(int64_t));
    for (int64_t i = 0; i < n; ++i)
        ++first[(ki[i].key >> shift) + 1];
    for (int k = 0; k < NBUCKET; ++k)
        first[k + 1] += first[k];
    int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * NBUCKET);
    memcpy(fill, first, sizeof(int64_t) * NBUCKET);
    keyidx *tmp = (keyidx *)malloc(sizeof(keyidx) * (size_t)n);
    for (int64_t i = 0; i < n; ++i)
        tmp[fill[ki[i].key >> shift]++] = ki[i];
#pragma omp parallel for schedule(dynamic, 1)
    for (int k = 0; k < NBUCKET; ++k)
        qsort(tmp + first[k], (size_t)(first[k + 1] - first[k]), sizeof(keyidx), cmp_keyidx);
    memcpy(ki, tmp, sizeof(keyidx) * (size_t)n);
    free(tmp); free(fill); free(first);
}

static void free_level(olevel *lv)
{
    free(lv->key); free(lv->start); free(lv->parent); free(lv->cstart);
    free(lv->near_ptr); free(lv->near_col); free(lv->far_ptr); free(lv->far_col);
    free(lv->small_ptr); free(lv->small_col);
    memset(lv, 0, sizeof(*lv));
}

void oracle_tree_free(otree *t)
{
    if (!t)
        return;
    for (int l = 0; l <= ORACLE_MAX_LEVELS; ++l)
        free_level(&t->lev[l]);
    free(t->cell); free(t->pkey); free(t->perm); free(t->rows_mark);
    free(t);
}

/* Divide: the box table of depth l, read off the permuted keys. */
static void divide(otree *t, int l)
{
    olevel *lv = &t->lev[l];
    int shift = t->D * (t->Lq - l);
    int64_t n = t->n, nb = 0;
    for (int64_t k = 0; k < n; ++k)
        if (k == 0 || (t->pkey[k] >> shift) != (t->pkey[k - 1] >> shift))
            ++nb;
    lv->nb = nb;
    lv->key = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)nb);
    lv->start = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nb + 1));
    lv->parent = (int64_t *)malloc(sizeof(int64_t) * (size_t)nb);
    int64_t r = 0;
    for (int64_t k = 0; k < n; ++k)
        if (k == 0 || (t->pkey[k] >> shift) != (t->pkey[k - 1] >> shift)) {
            lv->key[r] = t->pkey[k] >> shift;
            lv->start[r] = k;
            ++r;
        }
    lv->start[nb] = n;
    if (l > 0) {
        olevel *up = &t->lev[l - 1];
        up->cstart = (int64_t *)malloc(sizeof(int64_t) * (size_t)(up->nb + 1));
        int64_t P = -1;
        for (int64_t a = 0; a < nb; ++a) {
            if (a == 0 || (lv->key[a] >> t->D) != (lv->key[a - 1] >> t->D)) {
                ++P;
                up->cstart[P] = a;
            }
            lv->parent[a] = P;
        }
        up->cstart[up->nb] = nb;
    } else {
        lv->parent[0] = -1;
    }
}

static int64_t max_box(const olevel *lv)
{
    int64_t m = 0;
    for (int64_t a = 0; a < lv->nb; ++a)
        if (lv->start[a + 1] - lv->start[a] > m)
            m = lv->start[a + 1] - lv->start[a];
    return m;
}

/* New interactions at depth l from the near pairs of depth l-1, split into
 * near and far (reading R4).  Rows come out sorted because the parent's row is
 * sorted and the children of a box have consecutive ranks. */
static void new_interactions(otree *t, int l, double theta, int force_all_near, int all_interpolated,
                             int64_t rho, const uint8_t *only /* [nb] or NULL: rows to build (others stay empty) */)
{
    olevel *lv = &t->lev[l], *up = &t->lev[l - 1];
    int D = t->D;
    int64_t nb = lv->nb;
    lv->near_ptr = (int64_t *)calloc((size_t)(nb + 1), sizeof(int64_t));
    lv->far_ptr = (int64_t *)calloc((size_t)(nb + 1), sizeof(int64_t));
    lv->small_ptr = (int64_t *)calloc((size_t)(nb + 1), sizeof(int64_t));
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1) {
            for (int64_t a = 0; a < nb; ++a) {
                lv->near_ptr[a + 1] += lv->near_ptr[a];
                lv->far_ptr[a + 1] += lv->far_ptr[a];
                lv->small_ptr[a + 1] += lv->small_ptr[a];
            }
            lv->near_col = (int64_t *)malloc(sizeof(int64_t) * (size_t)(lv->near_ptr[nb] + 1));
            lv->far_col = (int64_t *)malloc(sizeof(int64_t) * (size_t)(lv->far_ptr[nb] + 1));
            lv->small_col = (int64_t *)malloc(sizeof(int64_t) * (size_t)(lv->small_ptr[nb] + 1));
        }
#pragma omp parallel for schedule(dynamic, 64)
        for (int64_t a = 0; a < nb; ++a) {
            int64_t ca[ORACLE_MAX_D], cb[ORACLE_MAX_D];
            deinterleave(lv->key[a], D, l, ca);
            int64_t P = lv->parent[a];
            int64_t nn = 0, nf = 0, ns = 0;
            int64_t *ncol = pass ? lv->near_col + lv->near_ptr[a] : NULL;
            int64_t *fcol = pass ? lv->far_col + lv->far_ptr[a] : NULL;
            int64_t *scol = pass ? lv->small_col + lv->small_ptr[a] : NULL;
            int64_t cnt_a = lv->start[a + 1] - lv->start[a];
            for (int64_t e = (only && !only[a]) ? up->near_ptr[P + 1] : up->near_ptr[P]; e < up->near_ptr[P + 1]; ++e) {
                int64_t Q = up->near_col[e];
                for (int64_t bq = up->cstart[Q]; bq < up->cstart[Q + 1]; ++bq) {
                    deinterleave(lv->key[bq], D, l, cb);
                    double d2 = 0.0;
                    for (int d = 0; d < D; ++d)
                        d2 += (double)((cb[d] - ca[d]) * (cb[d] - ca[d]));
                    /* smooth depth: adjacent pairs are interpolated too (Sec. 4.3) */
                    int is_far = all_interpolated || (!force_all_near && d2 >= theta * theta);
                    /* small field (Sec. 4.2): two boxes with few points are summed directly at
                     * this depth, whatever their distance, and the pair is not divided further */
                    int is_small = !force_all_near && rho > 0 &&
                                   cnt_a + (lv->start[bq + 1] - lv->start[bq]) <= rho;
                    if (is_small) {
                        if (pass) scol[ns] = bq;
                        ++ns;
                    } else if (is_far) {
                        if (pass) fcol[nf] = bq;
                        ++nf;
                    } else {
                        if (pass) ncol[nn] = bq;
                        ++nn;
                    }
                }
            }
            if (!pass) {
                lv->near_ptr[a + 1] = nn;
                lv->far_ptr[a + 1] = nf;
                lv->small_ptr[a + 1] = ns;
            }
        }
    }
}

/* Smoothness criterion with the O(1) bound of Sec. 4.3: the effective variance of a box of
 * edge l is at most D l^2 / (8 gamma^2) (variance <= l^2/4 per dimension), two boxes give
 * D l^2 / (4 gamma^2); adjacent pairs of a depth are interpolated when that is <= eta. */
int oracle_is_smooth_depth(double E, int depth, int D, double gamma, double eta_smooth)
{
    if (!(eta_smooth > 0.0) || !(gamma > 0.0))
        return 0;
    double l = E / ldexp(1.0, depth);
    return (double)D * l * l / (4.0 * gamma * gamma) <= eta_smooth;
}

/* Adaptive far-field rule of Sec. 4.3 on q = l^2 / (2 gamma^2), l the box edge of the depth:
 * nodes per dimension min(p, 3) if q <= 0.01 (the paper's min(r, 3^D) on a tensor grid),
 * p if 0.01 < q <= 5, and 0 (the far pairs of the depth are dropped) if q > 5. */
int oracle_adaptive_nodes(double E, int depth, double gamma, int p)
{
    double l = E / ldexp(1.0, depth);
    double q = l * l / (2.0 * gamma * gamma);
    if (q <= 0.01)
        return p < 3 ? p : 3;
    if (q <= 5.0)
        return p;
    return 0;
}

/* Per-dimension minimum of a point set and its largest extent, both in fp32 (R2). */
static float point_bounds(const float *X, int64_t n, int D, float *mn_out)
{
    float Ef = 0.0f;
    for (int d = 0; d < D; ++d) {
        float mn = X[d], mx = X[d];
        for (int64_t i = 1; i < n; ++i) {
            float v = X[i * D + d];
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
        volatile float ext = mx - mn;
        if (ext > Ef) Ef = ext;
        mn_out[d] = mn;
    }
    return Ef;
}

/* The points of one set in the cube anchored at alpha with edge Ef: cells and keys at the
 * quantisation depth (R2, R3), box order, and the box table of depth 0. */
static otree *partition_points(const float *X, int64_t n, int D, const float *alpha, float Ef)
{
    otree *t = (otree *)calloc(1, sizeof(otree));
    t->n = n;
    t->D = D;
    t->Lq = oracle_quant_depth(D);
    t->smooth_depth = -1;
    for (int d = 0; d < D; ++d)
        t->alpha[d] = (double)alpha[d];
    t->E = (double)Ef;
    t->s_f = Ef > 0.0f ? (float)(ldexp(1.0, t->Lq) / (double)Ef) : 0.0f;

    uint32_t cmax = (uint32_t)((1ull << t->Lq) - 1);
    t->cell = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)n * (size_t)D);
    keyidx *ki = (keyidx *)malloc(sizeof(keyidx) * (size_t)n);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int d = 0; d < D; ++d) {
            volatile float diff = X[i * D + d] - (float)t->alpha[d];
            volatile float u = diff * t->s_f;
            uint32_t c = (uint32_t)u;
            t->cell[i * D + d] = c > cmax ? cmax : c;
        }
        ki[i].key = interleave(&t->cell[i * D], D, t->Lq);
        ki[i].idx = i;
    }
    PROGRESS("cells and keys of %lld points", (long long)n);
    sort_keyidx(ki, n, D * t->Lq);
    PROGRESS("points sorted by (key, index)");
    t->pkey = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)n);
    t->perm = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
    for (int64_t k = 0; k < n; ++k) {
        t->pkey[k] = ki[k].key;
        t->perm[k] = ki[k].idx;
    }
    free(ki);
    divide(t, 0);
    return t;
}

otree *oracle_tree_build_ex(const float *X, int64_t n, int D, double theta, int64_t zeta, int max_depth,
                            int force_all_near, double gamma, double eta_smooth);
otree *oracle_tree_build_ex2(const float *X, int64_t n, int D, double theta, int64_t zeta, int max_depth,
                             int force_all_near, double gamma, double eta_smooth, int64_t rho);
otree *oracle_tree_build_rows(const float *X, int64_t n, int D, double theta, int64_t zeta, int max_depth,
                              int force_all_near, double gamma, double eta_smooth, const int64_t *rows, int64_t m);

/* Builds the partition and the interaction lists of Algorithm 1 (everything
 * that does not depend on b).  Returns NULL on bad arguments. */
otree *oracle_tree_build(const float *X, int64_t n, int D, double theta,
                         int64_t zeta, int max_depth, int force_all_near)
{
    return oracle_tree_build_ex(X, n, D, theta, zeta, max_depth, force_all_near, 0.0, 0.0);
}

/* The same with the smooth field of Sec. 4.3 (eta_smooth > 0): at the first depth whose boxes
 * pass the smoothness criterion every pair left is put on the far (interpolated) list, the
 * near list of that depth is empty and the loop of Algorithm 1 ends there. */
otree *oracle_tree_build_ex(const float *X, int64_t n, int D, double theta, int64_t zeta, int max_depth,
                            int force_all_near, double gamma, double eta_smooth)
{
    return oracle_tree_build_ex2(X, n, D, theta, zeta, max_depth, force_all_near, gamma, eta_smooth, 0);
}

/* for every box of depth l: does it hold one of the marked points?  selk is in box order */
static uint8_t *boxes_with_marked_points(const otree *t, int l, const uint8_t *selk)
{
    const olevel *lv = &t->lev[l];
    uint8_t *only = (uint8_t *)calloc((size_t)lv->nb, 1);
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < lv->nb; ++a)
        for (int64_t k = lv->start[a]; k < lv->start[a + 1]; ++k)
            if (selk[k]) {
                only[a] = 1;
                break;
            }
    return only;
}

static otree *tree_build_core(const float *X, int64_t n, int D, double theta, int64_t zeta, int max_depth,
                              int force_all_near, double gamma, double eta_smooth, int64_t rho,
                              const int64_t *rows, int64_t m)
{
    if (!X || n <= 0 || D < 1 || D > ORACLE_MAX_D || !(theta > 0.0) || zeta < 1)
        return NULL;
    /* enclosing cube: per-dim minimum, edge = largest extent (fp32, R2) */
    float mn[ORACLE_MAX_D];
    float Ef = point_bounds(X, n, D, mn);
    otree *t = partition_points(X, n, D, mn, Ef);
    t->gamma = eta_smooth > 0.0 ? gamma : 0.0;

    /* row subset: the points whose boxes get interaction rows, marked in box order */
    uint8_t *selk = NULL;
    if (rows) {
        uint8_t *sel = (uint8_t *)calloc((size_t)n, 1);
        for (int64_t a = 0; a < m; ++a)
            sel[rows[a]] = 1;
        selk = (uint8_t *)malloc((size_t)n);
        for (int64_t k = 0; k < n; ++k)
            selk[k] = sel[t->perm[k]];
        free(sel);
        t->rows_mark = selk;
    }

    /* depth 0: one box, one (near) interaction */
    olevel *root = &t->lev[0];
    root->near_ptr = (int64_t *)calloc(2, sizeof(int64_t));
    root->near_ptr[1] = 1;
    root->near_col = (int64_t *)calloc(1, sizeof(int64_t));
    root->far_ptr = (int64_t *)calloc(2, sizeof(int64_t));
    root->far_col = (int64_t *)calloc(1, sizeof(int64_t));
    root->small_ptr = (int64_t *)calloc(2, sizeof(int64_t));
    root->small_col = (int64_t *)calloc(1, sizeof(int64_t));

    int cap = t->Lq;
    if (max_depth > 0 && max_depth < cap) cap = max_depth;
    if (cap > ORACLE_MAX_LEVELS) cap = ORACLE_MAX_LEVELS;
    if (Ef == 0.0f) cap = 0; /* R6 */
    int l = 0;
    /* Algorithm 1: while interactions remain and the largest box is above zeta */
    while (t->lev[l].near_ptr[t->lev[l].nb] > 0 && max_box(&t->lev[l]) > zeta && l < cap) {
        ++l;
        divide(t, l);
        int smooth = !force_all_near && oracle_is_smooth_depth(t->E, l, D, gamma, eta_smooth);
        uint8_t *only = selk ? boxes_with_marked_points(t, l, selk) : NULL;
        new_interactions(t, l, theta, force_all_near, smooth, rho, only);
        free(only);
        PROGRESS("depth %d: %lld boxes, %lld near and %lld far pairs listed", l, (long long)t->lev[l].nb,
                 (long long)t->lev[l].near_ptr[t->lev[l].nb], (long long)t->lev[l].far_ptr[t->lev[l].nb]);
        if (smooth)
            t->smooth_depth = l;
    }
    t->L = l;
    return t;
}

/* The same with the small field of Sec. 4.2 (rho > 0): a pair of boxes created by a division whose
 * point counts add up to at most rho goes on the direct list of that depth. */
otree *oracle_tree_build_ex2(const float *X, int64_t n, int D, double theta, int64_t zeta, int max_depth,
                             int force_all_near, double gamma, double eta_smooth, int64_t rho)
{
    return tree_build_core(X, n, D, theta, zeta, max_depth, force_all_near, gamma, eta_smooth, rho, NULL, 0);
}

/* The tree for a subset of the rows of the product (Sec. 5, first paragraph: the error is measured
 * on a subset of rows): the partition is the full one, but interaction rows are built only for the
 * boxes that hold one of rows[0..m) (at every depth; all other rows stay empty), which is all that
 * oracle_f3m_apply_rows reads.  Without the small field (not offered here) a box with a row always
 * keeps its own pair until the smooth depth, so the loop of Algorithm 1 ends at the same depth as for
 * the full lists.  Rows out of range give NULL. */
otree *oracle_tree_build_rows(const float *X, int64_t n, int D, double theta, int64_t zeta, int max_depth,
                              int force_all_near, double gamma, double eta_smooth, const int64_t *rows, int64_t m)
{
    if (!rows || m <= 0)
        return NULL;
    for (int64_t a = 0; a < m; ++a)
        if (rows[a] < 0 || rows[a] >= n)
            return NULL;
    return tree_build_core(X, n, D, theta, zeta, max_depth, force_all_near, gamma, eta_smooth, 0, rows, m);
}

/* ---- introspection ---- */
int oracle_tree_depth(const otree *t) { return t->L; }
int oracle_tree_smooth_depth(const otree *t) { return t->smooth_depth; }
int oracle_tree_quant_depth(const otree *t) { return t->Lq; }
double oracle_tree_edge(const otree *t) { return t->E; }
void oracle_tree_alpha(const otree *t, double *alpha)
{
    for (int d = 0; d < t->D; ++d) alpha[d] = t->alpha[d];
}
int64_t oracle_tree_nboxes(const otree *t, int level) { return t->lev[level].nb; }
void oracle_tree_perm(const otree *t, int64_t *perm)
{
    memcpy(perm, t->perm, sizeof(int64_t) * (size_t)t->n);
}
/* key of every point at depth Lq, ORIGINAL order */
void oracle_tree_point_keys(const otree *t, uint64_t *keys)
{
    for (int64_t i = 0; i < t->n; ++i)
        keys[i] = interleave(&t->cell[i * t->D], t->D, t->Lq);
}
void oracle_tree_boxes(const otree *t, int level, uint64_t *keys, int64_t *starts)
{
    const olevel *lv = &t->lev[level];
    memcpy(keys, lv->key, sizeof(uint64_t) * (size_t)lv->nb);
    memcpy(starts, lv->start, sizeof(int64_t) * (size_t)(lv->nb + 1));
}
int64_t oracle_tree_list_size(const otree *t, int level, int kind)
{
    const olevel *lv = &t->lev[level];
    return kind == 2 ? lv->small_ptr[lv->nb] : kind ? lv->far_ptr[lv->nb] : lv->near_ptr[lv->nb];
}
void oracle_tree_list(const otree *t, int level, int kind, int64_t *row_ptr, int64_t *cols)
{
    const olevel *lv = &t->lev[level];
    const int64_t *ptr = kind == 2 ? lv->small_ptr : kind ? lv->far_ptr : lv->near_ptr;
    const int64_t *col = kind == 2 ? lv->small_col : kind ? lv->far_col : lv->near_col;
    memcpy(row_ptr, ptr, sizeof(int64_t) * (size_t)(lv->nb + 1));
    memcpy(cols, col, sizeof(int64_t) * (size_t)ptr[lv->nb]);
}
/* The row-major box index of Sec. 4.2 at a depth, per point, ORIGINAL order:
 * beta = sum_d 2^(depth*d) * cell_d  (d counted from 0). */
void oracle_beta(const otree *t, int level, uint64_t *beta)
{
    for (int64_t i = 0; i < t->n; ++i) {
        uint64_t bidx = 0;
        for (int d = 0; d < t->D; ++d)
            bidx += ((uint64_t)1 << (level * d)) * (uint64_t)(t->cell[i * t->D + d] >> (t->Lq - level));
        beta[i] = bidx;
    }
}

/* ------------------------------------------------------------------ */
/* far field and near field                                             */
/* ------------------------------------------------------------------ */
static int64_t ipow(int p, int D)
{
    int64_t r = 1;
    for (int d = 0; d < D; ++d) r *= p;
    return r;
}

/* centre of a box from its key (R7) */
static void box_centre(const otree *t, int level, uint64_t key, double *c)
{
    int64_t cell[ORACLE_MAX_D];
    deinterleave(key, t->D, level, cell);
    double l = t->E / ldexp(1.0, level);
    for (int d = 0; d < t->D; ++d)
        c[d] = t->alpha[d] + ((double)cell[d] + 0.5) * l;
}

/* node i of the grid of a box: centre + (l/2) * s_{i_d} in every dimension */
static void node_coords(const otree *t, int level, const double *centre, int p,
                        const double *s, int64_t i, double *x)
{
    double half = 0.5 * t->E / ldexp(1.0, level);
    for (int d = 0; d < t->D; ++d) {
        x[d] = centre[d] + half * s[i % p];
        i /= p;
    }
}

/* all r tensor-product Lagrange weights of one point of box `centre` */
static void point_weights(const otree *t, int level, const double *centre, int p,
                          const double *s, const float *x, double *Lw /* [r] */)
{
    int D = t->D;
    double half = 0.5 * t->E / ldexp(1.0, level);
    double L1[ORACLE_MAX_D][32];
    for (int d = 0; d < D; ++d) {
        double tt = ((double)x[d] - centre[d]) / half;
        oracle_lagrange_product(p, s, tt, L1[d]);
    }
    int64_t r = ipow(p, D);
    for (int64_t i = 0; i < r; ++i) {
        int64_t rem = i;
        double w = 1.0;
        for (int d = 0; d < D; ++d) {
            w *= L1[d][rem % p];
            rem /= p;
        }
        Lw[i] = w;
    }
}

/* v1 = L_Y b for one box: W[i] = sum_{j in box} L_i(t_j) b_j */
static void p2m_box(const otree *t, const float *X, const float *b, int level,
                    int64_t q, int p, const double *s, double *W, double *scratch)
{
    const olevel *lv = &t->lev[level];
    int64_t r = ipow(p, t->D);
    double centre[ORACLE_MAX_D];
    box_centre(t, level, lv->key[q], centre);
    for (int64_t i = 0; i < r; ++i) W[i] = 0.0;
    for (int64_t k = lv->start[q]; k < lv->start[q + 1]; ++k) {
        int64_t j = t->perm[k];
        point_weights(t, level, centre, p, s, X + j * t->D, scratch);
        for (int64_t i = 0; i < r; ++i) W[i] += scratch[i] * (double)b[j];
    }
}

/* Node weights W of every box of a depth (for the charge-conservation pin). */
void oracle_p2m_level(const otree *t, const float *X, const float *b, int p,
                      int level, double *W /* [nb*r] */)
{
    int64_t r = ipow(p, t->D);
    double s[32];
    oracle_cheb2_nodes(p, s);
#pragma omp parallel
    {
        double *scratch = (double *)malloc(sizeof(double) * (size_t)r);
#pragma omp for schedule(dynamic, 8)
        for (int64_t q = 0; q < t->lev[level].nb; ++q)
            p2m_box(t, X, b, level, q, p, s, W + q * r, scratch);
        free(scratch);
    }
}

/* y = F3M(X, b) following Algorithm 1.
 *   literal == 0: per depth, v1 of every source box is formed once, then
 *                 v2 of a target box is summed over its far row, then applied.
 *   literal == 1: every far pair is handled on its own, v1 -> v2 -> v, exactly
 *                 as a single far-field product is described (small inputs).
 * y is in ORIGINAL point order, fp64. */
int oracle_f3m_apply_ex(const otree *t, const float *X, double gamma, int p_all, int kernel_id, int kparam,
                        const float *b, double *y, int literal, int adaptive);
int oracle_f3m_apply_rows(const otree *t, const float *X, double gamma, int p_all, int kernel_id, int kparam,
                          const float *b, const int64_t *rows, int64_t m, double *y_rows, int adaptive);

int oracle_f3m_apply(const otree *t, const float *X, double gamma, int p,
                     int kernel_id, int kparam, const float *b, double *y, int literal)
{
    return oracle_f3m_apply_ex(t, X, gamma, p, kernel_id, kparam, b, y, literal, 0);
}

/* The rows of the product that are wanted: pos == NULL means every point (count == n, the value
 * of point k of the box order sits at index k); otherwise pos[0..count) are the box-order positions
 * of the wanted rows, ascending, and the value of pos[ip] sits at index ip. */
typedef struct {
    int64_t count;
    const int64_t *pos;
} rowsel;

/* first index ip whose position is >= k */
static int64_t rowsel_lower(const rowsel *S, int64_t k)
{
    if (!S->pos)
        return k;
    int64_t lo = 0, hi = S->count;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (S->pos[mid] < k) lo = mid + 1; else hi = mid;
    }
    return lo;
}

/* The target boxes of a depth that hold a wanted row, ascending; all boxes for pos == NULL. */
static int64_t *target_boxes(const olevel *lv, const rowsel *S, int64_t *count)
{
    int64_t *tb = (int64_t *)malloc(sizeof(int64_t) * (size_t)(S->pos ? S->count + 1 : lv->nb));
    int64_t nt = 0;
    if (!S->pos) {
        for (int64_t a = 0; a < lv->nb; ++a) tb[nt++] = a;
    } else {
        for (int64_t ip = 0; ip < S->count; ++ip) {
            /* box of position pos[ip]: last a with start[a] <= pos */
            int64_t lo = 0, hi = lv->nb;
            while (hi - lo > 1) {
                int64_t mid = lo + (hi - lo) / 2;
                if (lv->start[mid] <= S->pos[ip]) lo = mid; else hi = mid;
            }
            if (nt == 0 || tb[nt - 1] != lo) tb[nt++] = lo;
        }
    }
    *count = nt;
    return tb;
}

/* Algorithm 1 for the rows in S; ys[ip] receives the value of row ip of S.  The loops are the
 * same for every S: per depth v1 (of the source boxes that some wanted target's far row names),
 * v2 and v for the target boxes that hold a wanted row, then the exact sums. */
static void f3m_apply_core(const otree *t, const float *X, double gamma, int p_all, int kernel_id, int kparam,
                           const float *b, const rowsel *S, double *ys, int literal, int adaptive)
{
    int D = t->D;
    for (int64_t ip = 0; ip < S->count; ++ip) ys[ip] = 0.0;

    for (int l = 1; l <= t->L; ++l) {
        const olevel *lv = &t->lev[l];
        if (lv->far_ptr[lv->nb] == 0)
            continue;
        int p = adaptive ? oracle_adaptive_nodes(t->E, l, gamma, p_all) : p_all;
        if (p == 0)
            continue; /* interactions too far from each other are thrown away (Algorithm 1) */
        int64_t r = ipow(p, D);
        double s[32];
        oracle_cheb2_nodes(p, s);
        int64_t nt = 0;
        int64_t *tb = target_boxes(lv, S, &nt);
        /* v1 = L_Y b of the source boxes in use: slot[q] = row of W that holds box q, or -1 */
        double *W = NULL;
        int64_t *slot = NULL;
        if (!literal) {
            slot = (int64_t *)malloc(sizeof(int64_t) * (size_t)lv->nb);
            int64_t nsrc = 0;
            if (!S->pos) {
                for (int64_t q = 0; q < lv->nb; ++q) slot[q] = q;
                nsrc = lv->nb;
            } else {
                for (int64_t q = 0; q < lv->nb; ++q) slot[q] = -1;
                for (int64_t ai = 0; ai < nt; ++ai)
                    for (int64_t e = lv->far_ptr[tb[ai]]; e < lv->far_ptr[tb[ai] + 1]; ++e)
                        slot[lv->far_col[e]] = 0;
                for (int64_t q = 0; q < lv->nb; ++q)
                    if (slot[q] == 0) slot[q] = nsrc++;
            }
            W = (double *)malloc(sizeof(double) * (size_t)(nsrc > 0 ? nsrc : 1) * (size_t)r);
#pragma omp parallel
            {
                double *scratch = (double *)malloc(sizeof(double) * (size_t)r);
#pragma omp for schedule(dynamic, 8)
                for (int64_t q = 0; q < lv->nb; ++q)
                    if (slot[q] >= 0)
                        p2m_box(t, X, b, l, q, p, s, W + slot[q] * r, scratch);
                free(scratch);
            }
            PROGRESS("depth %d: node weights of %lld source boxes", l, (long long)nsrc);
        }
        if (literal) {
#pragma omp parallel
            {
                double *V = (double *)malloc(sizeof(double) * (size_t)r);
                double *Wq = (double *)malloc(sizeof(double) * (size_t)r);
                double *scratch = (double *)malloc(sizeof(double) * (size_t)r);
                double *xs = (double *)malloc(sizeof(double) * (size_t)r * D);
                double cp[ORACLE_MAX_D], cq[ORACLE_MAX_D], xq[ORACLE_MAX_D];
#pragma omp for schedule(dynamic, 1)
                for (int64_t ai = 0; ai < nt; ++ai) {
                    int64_t a = tb[ai];
                    const int64_t ip0 = rowsel_lower(S, lv->start[a]), ip1 = rowsel_lower(S, lv->start[a + 1]);
                    box_centre(t, l, lv->key[a], cp);
                    for (int64_t i = 0; i < r; ++i)
                        node_coords(t, l, cp, p, s, i, xs + i * D);
                    /* every far pair on its own: v1 of the source box, v2 = K v1, v = L_X^T v2 */
                    for (int64_t e = lv->far_ptr[a]; e < lv->far_ptr[a + 1]; ++e) {
                        int64_t q = lv->far_col[e];
                        p2m_box(t, X, b, l, q, p, s, Wq, scratch);
                        for (int64_t i = 0; i < r; ++i) V[i] = 0.0;
                        box_centre(t, l, lv->key[q], cq);
                        for (int64_t j = 0; j < r; ++j) {
                            node_coords(t, l, cq, p, s, j, xq);
                            for (int64_t i = 0; i < r; ++i)
                                V[i] += kernel_eval(kernel_id, kparam, gamma, D, xs + i * D, xq) * Wq[j];
                        }
                        for (int64_t ip = ip0; ip < ip1; ++ip) {
                            int64_t k = S->pos ? S->pos[ip] : ip;
                            point_weights(t, l, cp, p, s, X + t->perm[k] * D, scratch);
                            double acc = 0.0;
                            for (int64_t i = 0; i < r; ++i) acc += scratch[i] * V[i];
                            ys[ip] += acc;
                        }
                    }
                }
                free(V); free(Wq); free(scratch); free(xs);
            }
        } else {
            /* v2 = K v1 of every target box in use, summed over its far row: V[ai*r + i], i a node of
             * target box tb[ai].  Every V[i] is summed over (far pair, source node) in list order; with
             * few target boxes (a row subset) the nodes of a box are shared out between the threads in
             * `parts` ranges, which changes no sum. */
            double *V = (double *)malloc(sizeof(double) * (size_t)(nt > 0 ? nt : 1) * (size_t)r);
            int64_t parts = (S->pos && nt < 64) ? (r < 64 ? r : 64) : 1;
#pragma omp parallel
            {
                double *xs = (double *)malloc(sizeof(double) * (size_t)r * D);
                double cp[ORACLE_MAX_D], cq[ORACLE_MAX_D], xq[ORACLE_MAX_D];
#pragma omp for schedule(dynamic, 1)
                for (int64_t item = 0; item < nt * parts; ++item) {
                    int64_t ai = item / parts, part = item % parts;
                    int64_t i0 = r * part / parts, i1 = r * (part + 1) / parts;
                    int64_t a = tb[ai];
                    double *Va = V + ai * r;
                    box_centre(t, l, lv->key[a], cp);
                    for (int64_t i = i0; i < i1; ++i)
                        node_coords(t, l, cp, p, s, i, xs + i * D);
                    for (int64_t i = i0; i < i1; ++i) Va[i] = 0.0;
                    for (int64_t e = lv->far_ptr[a]; e < lv->far_ptr[a + 1]; ++e) {
                        int64_t q = lv->far_col[e];
                        const double *wq = W + slot[q] * r;
                        box_centre(t, l, lv->key[q], cq);
                        /* K_ij = k(s^p_i, s^q_j) */
                        for (int64_t j = 0; j < r; ++j) {
                            node_coords(t, l, cq, p, s, j, xq);
                            for (int64_t i = i0; i < i1; ++i)
                                Va[i] += kernel_eval(kernel_id, kparam, gamma, D, xs + i * D, xq) * wq[j];
                        }
                    }
                }
                free(xs);
            }
            /* v = L_X^T v2 */
#pragma omp parallel
            {
                double *scratch = (double *)malloc(sizeof(double) * (size_t)r);
                double cp[ORACLE_MAX_D];
#pragma omp for schedule(dynamic, 1)
                for (int64_t ai = 0; ai < nt; ++ai) {
                    int64_t a = tb[ai];
                    if (lv->far_ptr[a + 1] == lv->far_ptr[a])
                        continue;
                    const int64_t ip0 = rowsel_lower(S, lv->start[a]), ip1 = rowsel_lower(S, lv->start[a + 1]);
                    const double *Va = V + ai * r;
                    box_centre(t, l, lv->key[a], cp);
                    for (int64_t ip = ip0; ip < ip1; ++ip) {
                        int64_t k = S->pos ? S->pos[ip] : ip;
                        point_weights(t, l, cp, p, s, X + t->perm[k] * D, scratch);
                        double acc = 0.0;
                        for (int64_t i = 0; i < r; ++i) acc += scratch[i] * Va[i];
                        ys[ip] += acc;
                    }
                }
                free(scratch);
            }
            free(V);
        }
        free(W); free(slot); free(tb);
        PROGRESS("depth %d: far field of %lld target boxes", l, (long long)nt);
    }

    /* exact sums: the small-field pairs of every depth (Sec. 4.2) and the near-field
     * interactions that remain at the last depth */
    for (int l = 1; l <= t->L + 1; ++l) {
        const int last = l == t->L + 1;
        const olevel *lv = &t->lev[last ? t->L : l];
        const int64_t *ptr = last ? lv->near_ptr : lv->small_ptr;
        const int64_t *col = last ? lv->near_col : lv->small_col;
        if (!ptr || ptr[lv->nb] == 0)
            continue;
        int64_t nt = 0;
        int64_t *tb = target_boxes(lv, S, &nt);
#pragma omp parallel for schedule(dynamic, 4)
        for (int64_t ai = 0; ai < nt; ++ai) {
            int64_t a = tb[ai];
            double xi[ORACLE_MAX_D], xj[ORACLE_MAX_D];
            const int64_t ip0 = rowsel_lower(S, lv->start[a]), ip1 = rowsel_lower(S, lv->start[a + 1]);
            for (int64_t ip = ip0; ip < ip1; ++ip) {
                int64_t k = S->pos ? S->pos[ip] : ip;
                int64_t i = t->perm[k];
                for (int d = 0; d < D; ++d) xi[d] = (double)X[i * D + d];
                double acc = 0.0;
                for (int64_t e = ptr[a]; e < ptr[a + 1]; ++e) {
                    int64_t q = col[e];
                    for (int64_t kk = lv->start[q]; kk < lv->start[q + 1]; ++kk) {
                        int64_t j = t->perm[kk];
                        for (int d = 0; d < D; ++d) xj[d] = (double)X[j * D + d];
                        acc += kernel_eval(kernel_id, kparam, gamma, D, xi, xj) * (double)b[j];
                    }
                }
                ys[ip] += acc;
            }
        }
        free(tb);
    }
}

/* adaptive != 0: the node count of every depth follows oracle_adaptive_nodes (Sec. 4.3,
 * adaptive far-field approximation; a depth with 0 nodes contributes nothing). */
int oracle_f3m_apply_ex(const otree *t, const float *X, double gamma, int p_all, int kernel_id, int kparam,
                        const float *b, double *y, int literal, int adaptive)
{
    if (!t || !X || !b || !y || p_all < 2 || p_all > 32)
        return 1;
    if (t->gamma != 0.0 && t->gamma != gamma)
        return 2; /* the smooth rule of the tree was evaluated with another lengthscale */
    if (t->rows_mark)
        return 3; /* the tree holds the interaction rows of a row subset only */
    int64_t n = t->n;
    double *ys = (double *)malloc(sizeof(double) * (size_t)n); /* box order */
    rowsel S = { n, NULL };
    f3m_apply_core(t, X, gamma, p_all, kernel_id, kparam, b, &S, ys, literal, adaptive);
    /* back to the caller's order */
    for (int64_t k = 0; k < n; ++k)
        y[t->perm[k]] = ys[k];
    free(ys);
    return 0;
}

typedef struct {
    int64_t row, pos;
} rowpos;

static int cmp_rowpos(const void *a, const void *b)
{
    const rowpos *p = (const rowpos *)a, *q = (const rowpos *)b;
    return p->row < q->row ? -1 : (p->row > q->row);
}

/* The rows rows[0..m) of the same product (Sec. 5, first paragraph: results are compared on a
 * subset of rows): y_rows[a] = row rows[a] of oracle_f3m_apply_ex.  The steps are those of the
 * full product, run over the boxes that hold a wanted row and over the source boxes their far rows
 * name; every sum that reaches a wanted row is formed in the same order, so the values are the
 * same bits.  Works on a full tree and on a tree of oracle_tree_build_rows whose subset holds
 * every wanted row. */
int oracle_f3m_apply_rows(const otree *t, const float *X, double gamma, int p_all, int kernel_id, int kparam,
                          const float *b, const int64_t *rows, int64_t m, double *y_rows, int adaptive)
{
    if (!t || !X || !b || !y_rows || !rows || m < 0 || p_all < 2 || p_all > 32)
        return 1;
    if (t->gamma != 0.0 && t->gamma != gamma)
        return 2;
    int64_t n = t->n;
    for (int64_t a = 0; a < m; ++a)
        if (rows[a] < 0 || rows[a] >= n)
            return 1;
    /* box-order positions of the wanted rows, ascending, duplicates merged */
    uint8_t *sel = (uint8_t *)calloc((size_t)n, 1);
    for (int64_t a = 0; a < m; ++a)
        sel[rows[a]] = 1;
    int64_t count = 0;
    for (int64_t i = 0; i < n; ++i)
        count += sel[i];
    int64_t *pos = (int64_t *)malloc(sizeof(int64_t) * (size_t)(count + 1));
    rowpos *rp = (rowpos *)malloc(sizeof(rowpos) * (size_t)(count + 1));
    int64_t c = 0;
    int bad = 0;
    for (int64_t k = 0; k < n; ++k)
        if (sel[t->perm[k]]) {
            if (t->rows_mark && !t->rows_mark[k])
                bad = 1; /* the tree has no interaction rows for the box of this point */
            pos[c] = k;
            rp[c].row = t->perm[k];
            rp[c].pos = c;
            ++c;
        }
    free(sel);
    if (bad) {
        free(pos); free(rp);
        return 3;
    }
    double *ys = (double *)malloc(sizeof(double) * (size_t)(count + 1));
    rowsel S = { count, pos };
    f3m_apply_core(t, X, gamma, p_all, kernel_id, kparam, b, &S, ys, 0, adaptive);
    qsort(rp, (size_t)count, sizeof(rowpos), cmp_rowpos);
    for (int64_t a = 0; a < m; ++a) {
        int64_t lo = 0, hi = count;
        while (hi - lo > 1) {
            int64_t mid = lo + (hi - lo) / 2;
            if (rp[mid].row <= rows[a]) lo = mid; else hi = mid;
        }
        y_rows[a] = ys[rp[lo].pos];
    }
    free(ys); free(pos); free(rp);
    return 0;
}

/* ------------------------------------------------------------------ */
/* two point sets: v = K(X, Y) b                                        */
/* ------------------------------------------------------------------ */
/* Sec. 3 states the method for a kernel evaluated on two data matrices X (targets, n_x rows)
 * and Y (sources, n_y rows, b holds one weight per row of Y); Algorithm 1 keeps one treecode per
 * set.  Readings for X != Y:
 *   R8   both sets get a cube of the SAME edge E = max(largest extent of X, largest extent of Y)
 *        (Sec. 3, enclosing formula), each anchored at its own per-dimension minimum (the alpha
 *        of the box-index formula of Sec. 4.2 is the minimum of the set that is divided).  The
 *        two grids have equal box edges at every depth and are shifted against each other by
 *        alpha^Y - alpha^X.
 *   R9   far iff |centre_y - centre_x| >= theta * l.  In units of l the centre difference of
 *        source cell c' and target cell c is (c'_d - c_d) + u_d with u_d = (alpha^Y_d -
 *        alpha^X_d) / l, so far iff  sum_d ((c'_d - c_d) + u_d)^2 >= theta^2.  This decision is
 *        taken in fp64 with u_d = ((alpha^Y_d - alpha^X_d) / E) * 2^depth, the sum taken in the
 *        order d = 0..D-1, every operation rounded on its own.  With X == Y it is R4.
 *   R10  Algorithm 1 divides while interactions remain, the largest box of tau_x is above zeta
 *        AND the largest box of tau_y is above zeta; depth caps as in R6.
 *   R11  small field: |B_p^X| + |B_q^Y| <= rho.  Smooth field and adaptive rule: functions of
 *        the common box edge, unchanged.
 * Lists are stored by target box (a box of tau_x); the columns are ranks of boxes of tau_y. */
typedef struct {
    int64_t *near_ptr, *near_col, *far_ptr, *far_col, *small_ptr, *small_col;
} olists;

typedef struct {
    otree *tx, *ty; /* the two partitions; their own list fields stay unused */
    int D, L, smooth_depth;
    double E, gamma, theta;
    olists lev[ORACLE_MAX_LEVELS + 1];
} otree2;

/* y_i = sum_j k(x_i, y_j) b_j for the rows of X listed in rows[0..m) (NULL: all rows, m = n_x) */
void oracle_rows_xy(const float *X, int64_t nx, const float *Y, int64_t ny, int D, double gamma,
                    int kernel_id, int kparam, const float *b, const int64_t *rows, int64_t m, double *y)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t a = 0; a < m; ++a) {
        int64_t i = rows ? rows[a] : a;
        double xi[ORACLE_MAX_D], yj[ORACLE_MAX_D];
        for (int d = 0; d < D; ++d)
            xi[d] = (double)X[i * D + d];
        double acc = 0.0;
        for (int64_t j = 0; j < ny; ++j) {
            for (int d = 0; d < D; ++d)
                yj[d] = (double)Y[j * D + d];
            acc += kernel_eval(kernel_id, kparam, gamma, D, xi, yj) * (double)b[j];
        }
        y[a] = acc;
    }
    (void)nx;
}

void oracle_tree2_free(otree2 *t)
{
    if (!t)
        return;
    for (int l = 0; l <= ORACLE_MAX_LEVELS; ++l) {
        olists *ls = &t->lev[l];
        free(ls->near_ptr); free(ls->near_col); free(ls->far_ptr); free(ls->far_col);
        free(ls->small_ptr); free(ls->small_col);
    }
    oracle_tree_free(t->tx);
    oracle_tree_free(t->ty);
    free(t);
}

/* squared centre distance of source cell cb and target cell ca in units of the box edge (R9) */
static double centre_dist2(int D, const int64_t *ca, const int64_t *cb, const double *u)
{
    double d2 = 0.0;
    for (int d = 0; d < D; ++d) {
        volatile double o = (double)(cb[d] - ca[d]) + u[d];
        volatile double sq = o * o;
        d2 = d2 + sq;
    }
    return d2;
}

/* grid shift of a depth in units of its box edge (R9) */
static void grid_shift(const otree2 *t, int l, double *u)
{
    for (int d = 0; d < t->D; ++d) {
        volatile double diff = t->ty->alpha[d] - t->tx->alpha[d];
        volatile double q = t->E > 0.0 ? diff / t->E : 0.0;
        u[d] = q * ldexp(1.0, l);
    }
}

/* New interactions at depth l: children of a target box's parent's near partners, split three
 * ways (small first, then far, else near), as for one point set. */
static void new_interactions2(otree2 *t, int l, int force_all_near, int all_interpolated, int64_t rho)
{
    const olevel *xv = &t->tx->lev[l], *xu = &t->tx->lev[l - 1];
    const olevel *yv = &t->ty->lev[l], *yu = &t->ty->lev[l - 1];
    olists *ls = &t->lev[l], *up = &t->lev[l - 1];
    int D = t->D;
    int64_t nb = xv->nb;
    double u[ORACLE_MAX_D];
    grid_shift(t, l, u);
    const double theta2 = t->theta * t->theta;
    ls->near_ptr = (int64_t *)calloc((size_t)(nb + 1), sizeof(int64_t));
    ls->far_ptr = (int64_t *)calloc((size_t)(nb + 1), sizeof(int64_t));
    ls->small_ptr = (int64_t *)calloc((size_t)(nb + 1), sizeof(int64_t));
    (void)xu;
    for (int pass = 0; pass < 2; ++pass) {
        if (pass == 1) {
            for (int64_t a = 0; a < nb; ++a) {
                ls->near_ptr[a + 1] += ls->near_ptr[a];
                ls->far_ptr[a + 1] += ls->far_ptr[a];
                ls->small_ptr[a + 1] += ls->small_ptr[a];
            }
            ls->near_col = (int64_t *)malloc(sizeof(int64_t) * (size_t)(ls->near_ptr[nb] + 1));
            ls->far_col = (int64_t *)malloc(sizeof(int64_t) * (size_t)(ls->far_ptr[nb] + 1));
            ls->small_col = (int64_t *)malloc(sizeof(int64_t) * (size_t)(ls->small_ptr[nb] + 1));
        }
#pragma omp parallel for schedule(dynamic, 64)
        for (int64_t a = 0; a < nb; ++a) {
            int64_t ca[ORACLE_MAX_D], cb[ORACLE_MAX_D];
            deinterleave(xv->key[a], D, l, ca);
            int64_t P = xv->parent[a];
            int64_t nn = 0, nf = 0, ns = 0;
            int64_t *ncol = pass ? ls->near_col + ls->near_ptr[a] : NULL;
            int64_t *fcol = pass ? ls->far_col + ls->far_ptr[a] : NULL;
            int64_t *scol = pass ? ls->small_col + ls->small_ptr[a] : NULL;
            int64_t cnt_a = xv->start[a + 1] - xv->start[a];
            for (int64_t e = up->near_ptr[P]; e < up->near_ptr[P + 1]; ++e) {
                int64_t Q = up->near_col[e];
                for (int64_t bq = yu->cstart[Q]; bq < yu->cstart[Q + 1]; ++bq) {
                    deinterleave(yv->key[bq], D, l, cb);
                    int is_far = all_interpolated ||
                                 (!force_all_near && centre_dist2(D, ca, cb, u) >= theta2);
                    int is_small = !force_all_near && rho > 0 &&
                                   cnt_a + (yv->start[bq + 1] - yv->start[bq]) <= rho;
                    if (is_small) {
                        if (pass) scol[ns] = bq;
                        ++ns;
                    } else if (is_far) {
                        if (pass) fcol[nf] = bq;
                        ++nf;
                    } else {
                        if (pass) ncol[nn] = bq;
                        ++nn;
                    }
                }
            }
            if (!pass) {
                ls->near_ptr[a + 1] = nn;
                ls->far_ptr[a + 1] = nf;
                ls->small_ptr[a + 1] = ns;
            }
        }
    }
}

/* Partitions of both sets and the interaction lists of Algorithm 1 for K(X, Y).  Arguments as
 * oracle_tree_build_ex2.  Returns NULL on bad arguments. */
otree2 *oracle_tree2_build(const float *X, int64_t nx, const float *Y, int64_t ny, int D, double theta,
                           int64_t zeta, int max_depth, int force_all_near, double gamma, double eta_smooth,
                           int64_t rho)
{
    if (!X || !Y || nx <= 0 || ny <= 0 || D < 1 || D > ORACLE_MAX_D || !(theta > 0.0) || zeta < 1)
        return NULL;
    otree2 *t = (otree2 *)calloc(1, sizeof(otree2));
    t->D = D;
    t->theta = theta;
    t->smooth_depth = -1;
    t->gamma = eta_smooth > 0.0 ? gamma : 0.0;
    /* cubes of a common edge, each anchored at its own minimum (R8) */
    float ax[ORACLE_MAX_D], ay[ORACLE_MAX_D];
    float Ex = point_bounds(X, nx, D, ax), Ey = point_bounds(Y, ny, D, ay);
    float Ef = Ex > Ey ? Ex : Ey;
    t->tx = partition_points(X, nx, D, ax, Ef);
    t->ty = partition_points(Y, ny, D, ay, Ef);
    t->E = (double)Ef;

    /* depth 0: one box per set, one (near) interaction */
    olists *root = &t->lev[0];
    root->near_ptr = (int64_t *)calloc(2, sizeof(int64_t));
    root->near_ptr[1] = 1;
    root->near_col = (int64_t *)calloc(1, sizeof(int64_t));
    root->far_ptr = (int64_t *)calloc(2, sizeof(int64_t));
    root->far_col = (int64_t *)calloc(1, sizeof(int64_t));
    root->small_ptr = (int64_t *)calloc(2, sizeof(int64_t));
    root->small_col = (int64_t *)calloc(1, sizeof(int64_t));

    int cap = t->tx->Lq;
    if (max_depth > 0 && max_depth < cap) cap = max_depth;
    if (cap > ORACLE_MAX_LEVELS) cap = ORACLE_MAX_LEVELS;
    if (Ef == 0.0f) cap = 0;
    int l = 0;
    /* Algorithm 1: while interactions remain and the largest box of either tree is above zeta (R10) */
    while (t->lev[l].near_ptr[t->tx->lev[l].nb] > 0 && max_box(&t->tx->lev[l]) > zeta &&
           max_box(&t->ty->lev[l]) > zeta && l < cap) {
        ++l;
        divide(t->tx, l);
        divide(t->ty, l);
        int smooth = !force_all_near && oracle_is_smooth_depth(t->E, l, D, gamma, eta_smooth);
        new_interactions2(t, l, force_all_near, smooth, rho);
        if (smooth)
            t->smooth_depth = l;
    }
    t->L = l;
    t->tx->L = t->ty->L = l;
    return t;
}

int oracle_tree2_depth(const otree2 *t) { return t->L; }
int oracle_tree2_smooth_depth(const otree2 *t) { return t->smooth_depth; }
double oracle_tree2_edge(const otree2 *t) { return t->E; }
/* the partition of one set (side 0: X, 1: Y) for the single-set introspection calls
 * (perm, point keys, boxes, alpha, beta); owned by the two-set tree */
const otree *oracle_tree2_side(const otree2 *t, int side) { return side ? t->ty : t->tx; }
int64_t oracle_tree2_list_size(const otree2 *t, int level, int kind)
{
    const olists *ls = &t->lev[level];
    int64_t nb = t->tx->lev[level].nb;
    return kind == 2 ? ls->small_ptr[nb] : kind ? ls->far_ptr[nb] : ls->near_ptr[nb];
}
void oracle_tree2_list(const otree2 *t, int level, int kind, int64_t *row_ptr, int64_t *cols)
{
    const olists *ls = &t->lev[level];
    int64_t nb = t->tx->lev[level].nb;
    const int64_t *ptr = kind == 2 ? ls->small_ptr : kind ? ls->far_ptr : ls->near_ptr;
    const int64_t *col = kind == 2 ? ls->small_col : kind ? ls->far_col : ls->near_col;
    memcpy(row_ptr, ptr, sizeof(int64_t) * (size_t)(nb + 1));
    memcpy(cols, col, sizeof(int64_t) * (size_t)ptr[nb]);
}

/* v = F3M(X, Y, b) following Algorithm 1: per depth v1 = L_Y b of every source box (tau_y),
 * v2 = sum over the far row of K v1 at the nodes of the target box (tau_x), v += L_X^T v2; then
 * the direct sums over the small-field pairs of every depth and the near pairs of the last one.
 * y has n_x entries in the ORIGINAL order of X, fp64. */
int oracle_f3m2_apply(const otree2 *t, const float *X, const float *Y, double gamma, int p_all, int kernel_id,
                      int kparam, const float *b, double *y, int adaptive)
{
    if (!t || !X || !Y || !b || !y || p_all < 2 || p_all > 32)
        return 1;
    if (t->gamma != 0.0 && t->gamma != gamma)
        return 2;
    const otree *tx = t->tx, *ty = t->ty;
    int D = t->D;
    int64_t nx = tx->n;
    double *ys = (double *)calloc((size_t)nx, sizeof(double)); /* box order of X */

    for (int l = 1; l <= t->L; ++l) {
        const olists *ls = &t->lev[l];
        const olevel *xv = &tx->lev[l], *yv = &ty->lev[l];
        if (ls->far_ptr[xv->nb] == 0)
            continue;
        int p = adaptive ? oracle_adaptive_nodes(t->E, l, gamma, p_all) : p_all;
        if (p == 0)
            continue;
        int64_t r = ipow(p, D);
        double s[32];
        oracle_cheb2_nodes(p, s);
        double *W = (double *)malloc(sizeof(double) * (size_t)yv->nb * (size_t)r);
        oracle_p2m_level(ty, Y, b, p, l, W);
#pragma omp parallel
        {
            double *V = (double *)malloc(sizeof(double) * (size_t)r);
            double *scratch = (double *)malloc(sizeof(double) * (size_t)r);
            double *xs = (double *)malloc(sizeof(double) * (size_t)r * D);
            double cp[ORACLE_MAX_D], cq[ORACLE_MAX_D], xq[ORACLE_MAX_D];
#pragma omp for schedule(dynamic, 4)
            for (int64_t a = 0; a < xv->nb; ++a) {
                if (ls->far_ptr[a + 1] == ls->far_ptr[a])
                    continue;
                box_centre(tx, l, xv->key[a], cp);
                for (int64_t i = 0; i < r; ++i)
                    node_coords(tx, l, cp, p, s, i, xs + i * D);
                for (int64_t i = 0; i < r; ++i) V[i] = 0.0;
                for (int64_t e = ls->far_ptr[a]; e < ls->far_ptr[a + 1]; ++e) {
                    int64_t q = ls->far_col[e];
                    const double *wq = W + q * r;
                    box_centre(ty, l, yv->key[q], cq);
                    for (int64_t j = 0; j < r; ++j) {
                        node_coords(ty, l, cq, p, s, j, xq);
                        for (int64_t i = 0; i < r; ++i)
                            V[i] += kernel_eval(kernel_id, kparam, gamma, D, xs + i * D, xq) * wq[j];
                    }
                }
                for (int64_t k = xv->start[a]; k < xv->start[a + 1]; ++k) {
                    point_weights(tx, l, cp, p, s, X + tx->perm[k] * D, scratch);
                    double acc = 0.0;
                    for (int64_t i = 0; i < r; ++i) acc += scratch[i] * V[i];
                    ys[k] += acc;
                }
            }
            free(V); free(scratch); free(xs);
        }
        free(W);
    }

    for (int l = 1; l <= t->L + 1; ++l) {
        const int last = l == t->L + 1;
        const int lev = last ? t->L : l;
        const olists *ls = &t->lev[lev];
        const olevel *xv = &tx->lev[lev], *yv = &ty->lev[lev];
        const int64_t *ptr = last ? ls->near_ptr : ls->small_ptr;
        const int64_t *col = last ? ls->near_col : ls->small_col;
        if (!ptr || ptr[xv->nb] == 0)
            continue;
#pragma omp parallel for schedule(dynamic, 4)
        for (int64_t a = 0; a < xv->nb; ++a) {
            double xi[ORACLE_MAX_D], yj[ORACLE_MAX_D];
            for (int64_t k = xv->start[a]; k < xv->start[a + 1]; ++k) {
                int64_t i = tx->perm[k];
                for (int d = 0; d < D; ++d) xi[d] = (double)X[i * D + d];
                double acc = 0.0;
                for (int64_t e = ptr[a]; e < ptr[a + 1]; ++e) {
                    int64_t q = col[e];
                    for (int64_t kk = yv->start[q]; kk < yv->start[q + 1]; ++kk) {
                        int64_t j = ty->perm[kk];
                        for (int d = 0; d < D; ++d) yj[d] = (double)Y[j * D + d];
                        acc += kernel_eval(kernel_id, kparam, gamma, D, xi, yj) * (double)b[j];
                    }
                }
                ys[k] += acc;
            }
        }
    }
    for (int64_t k = 0; k < nx; ++k)
        y[tx->perm[k]] = ys[k];
    free(ys);
    return 0;
}
