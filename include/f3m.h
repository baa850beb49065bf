/*
 * f3m.h - C ABI of the MI355X (gfx950) F3M kernel matrix-vector product.
 *
 * The library computes y = K(X,X) b for the Gaussian kernel
 * k(x,y) = exp(-|x-y|^2 / (2 gamma^2)) (arXiv 2202.01085, Sec. 5, first
 * paragraph) on n points in D <= 7 dimensions, either exactly (direct_kmvm)
 * or with the hierarchical F3M approximation (f3m_plan + f3m_kmvm) of
 * Sec. 3 and Appendix E, Algorithm 1.  The *_xy entry points do the same for
 * two point sets, v = K(X,Y) b, the general form of Sec. 3.
 *
 * Conventions shared by every entry point
 *   - X, b, y are DEVICE pointers (fp32).  X is n x D row-major, the paper's
 *     X in R^{n x D} (Sec. 1, "Notations").  b and y have n entries in the
 *     caller's point order.  Introspection calls copy to HOST buffers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Work is enqueued on it; see each call for whether it synchronises.
 *   - Every call returns an f3m_status; nothing throws or aborts across the
 *     boundary.  f3m_last_error() gives a thread-local message for the last
 *     failing call of the calling thread.
 *   - The caller owns X, b, y.  A plan owns all of its device buffers and
 *     keeps no reference to X after f3m_plan returns.  Device memory of the
 *     library is cached by a pool (see f3m_destroy, f3m_trim_memory).
 *   - There is no CPU fallback: without a HIP device every compute call
 *     returns F3M_ERR_HIP.
 */
#ifndef F3M_H
#define F3M_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define F3M_MAX_DIM 7
#define F3M_MAX_LEVELS 20

typedef struct f3m_plan_s f3m_plan_t; /* opaque */

typedef enum {
    F3M_OK = 0,
    F3M_ERR_INVALID_ARG = 1, /* null pointer, n < 0, D outside [1,7], interp_nodes < 2,
                                lengthscale or eta not finite and positive, bad level/kind */
    F3M_ERR_NONFINITE = 2,   /* NaN or Inf among the coordinates */
    F3M_ERR_UNSUPPORTED = 3, /* n >= 2^31, interp_nodes > 8, interp_nodes^D above the node cap (4096), or an eta
                                so large that the per-depth factor tables of the M2L exceed 64 KB (roughly
                                eta > 25 .. 100, depending on D and interp_nodes) */
    F3M_ERR_OOM = 4,         /* a device allocation failed */
    F3M_ERR_HIP = 5,         /* any other HIP runtime error (message in f3m_last_error) */
    F3M_ERR_BREAKDOWN = 6    /* f3m_cg_solve: a search direction with p.(K + lambda I)p <= 0 */
} f3m_status;

typedef struct {
    int32_t leaf_max;       /* zeta of Algorithm 1: divide while the LARGEST box holds more
                               points than this; 0 = library default (128) */
    int32_t max_depth;      /* cap on the number of divisions; 0 = the quantisation depth */
    int32_t force_all_near; /* test hook: classify every pair as near, so that the result
                               must equal direct_kmvm */
    int32_t overlap;        /* 1: the near field runs on a second stream of the plan, concurrently with
                               the far field (measured gain about 4 %); 0 (default): everything in order
                               on the caller's stream (per-kernel timings are then undisturbed) */
    float eta_smooth;       /* smooth field of Sec. 4.3 ("Smoothness criteria"): once the boxes of a depth
                               satisfy D l^2 / (4 lengthscale^2) <= eta_smooth (l = box edge, the O(1) bound
                               on the effective variance of two boxes) every pair left at that depth,
                               adjacent and self pairs included, is interpolated like a far pair and the
                               division stops: no near field remains.  0 (default) = off; the paper uses
                               0.1 .. 0.5.  Must be finite and >= 0. */
    int32_t adaptive_far;   /* adaptive far-field approximation of Sec. 4.3: with q = l^2 / (2 lengthscale^2)
                               a depth uses min(interp_nodes, 3) nodes per dimension if q <= 0.01,
                               interp_nodes if q <= 5, and its far pairs are dropped if q > 5.
                               0 (default) = every depth uses interp_nodes. */
    int32_t small_field;    /* small field of Sec. 4.2 ("Handling boxes with few points"): rho >= 0.  A pair of
                               boxes created by a division whose point counts add up to at most rho is
                               summed directly (exactly) at that depth, whatever its distance, and is not
                               divided further.  0 (default) = off; the paper suggests rho = 2 * nodes per
                               box. */
    int32_t route_min_points; /* a point set with at least this many points moves b, y and its own coordinates
                               between the caller's order and the box order in three streaming passes through
                               LDS instead of one random gather or scatter (same values, bit for bit); 0 =
                               library default (2^24: below it the caches hold the vectors).  A smaller value
                               lets tests reach that path on small inputs. */
} f3m_options;

typedef struct {
    int64_t n;
    int32_t D;
    int32_t interp_nodes;   /* p, nodes per dimension */
    int32_t nodes_per_box;  /* r = p^D */
    int32_t depth;          /* L: divisions actually made (near field is evaluated at depth L) */
    int32_t quant_depth;    /* depth at which cells are quantised once (keys have D*quant_depth bits) */
    int32_t far_threshold;  /* T = ceil(eta^2): a pair is far iff the squared integer cell offset >= T */
    float edge;             /* E, edge of the enclosing cube */
    float scale;            /* fp32 factor 2^quant_depth / E used for the cells */
    float alpha[F3M_MAX_DIM];                  /* per-dimension minimum (cube anchor) */
    int64_t nboxes[F3M_MAX_LEVELS + 1];        /* occupied boxes per depth 0..L */
    int64_t max_box[F3M_MAX_LEVELS + 1];       /* largest box per depth */
    int64_t near_pairs[F3M_MAX_LEVELS + 1];    /* ordered near pairs per depth */
    int64_t far_pairs[F3M_MAX_LEVELS + 1];     /* ordered far pairs per depth */
    int64_t far_point_pairs[F3M_MAX_LEVELS + 1]; /* per depth: sum of |p||q| over the far pairs; with
                                                  near_point_pairs they add up to n*n */
    int64_t near_point_pairs;                  /* point pairs evaluated exactly: sum of |p||q| over the
                                                  near pairs of depth L */
    int64_t device_bytes;                      /* device memory held by the plan */
    int32_t smooth_depth;                      /* depth whose adjacent pairs are interpolated (smooth
                                                  field), -1 if none */
    int32_t level_nodes[F3M_MAX_LEVELS + 1];   /* nodes per dimension used at each depth 1..L (0: the far
                                                  pairs of the depth are dropped by the adaptive rule) */
    int64_t small_pairs[F3M_MAX_LEVELS + 1];   /* ordered small-field pairs per depth */
    int64_t small_point_pairs[F3M_MAX_LEVELS + 1]; /* their point pairs; far + small + near = n*n */
} f3m_info;

typedef struct {
    /* milliseconds of the most recent f3m_plan / f3m_kmvm on this plan */
    float bbox_keys, sort, gather, boxes, lists, tables, plan_total;
    float permute_in, p2p, p2m, m2l, l2p, permute_out, kmvm_total;
} f3m_times;

/*
 * f3m_plan - everything of Algorithm 1 (Appendix E) that does not depend on b:
 * the enclosing cube (Sec. 3 "Enclosing and partitioning the data"), the box of
 * every point (Sec. 4.2 box-index formula), the grouping permutation (Sec. 4.1
 * "In-place grouping data on boxes"; here one stable radix sort of 32-bit
 * interleaved keys), the occupied-box tables per depth (Sec. 4.2 "Removing empty
 * boxes"), the near/far interaction lists per depth (Sec. 3 "Far and near-field
 * interactions", Sec. 4.1 "Ensuring interactions are sorted") and the
 * node-to-node kernel tables (Sec. 3 "Interpolating k(x,y)", step 2 of Fig. 4).
 *
 *   X            device, n x D row-major fp32; read only during the call
 *   n            number of points, 0 <= n < 2^31
 *   D            1..7
 *   lengthscale  gamma > 0
 *   interp_nodes 2 <= p <= 8 Chebyshev nodes of the second kind per dimension, with p^D <= 4096
 *                (p = 4 in 3-D is the paper's r = 64); F3M_ERR_UNSUPPORTED above either limit
 *   eta          far-field distance ratio theta: boxes are far iff the distance
 *                of their centres is >= theta * (box edge); the paper uses 2.
 *                (NOT the paper's smooth-field limit: that is f3m_options.eta_smooth.)
 *   stream       the call enqueues on it and synchronises it several times
 *   plan_out     receives the plan; NULL on error.  n == 0 gives an empty plan.
 */
f3m_status f3m_plan(const float *X, int64_t n, int D, float lengthscale, int interp_nodes,
                    float eta, void *stream, f3m_plan_t **plan_out);

/* f3m_plan with explicit options (opt == NULL: defaults). */
f3m_status f3m_plan_ex(const float *X, int64_t n, int D, float lengthscale, int interp_nodes,
                       float eta, const f3m_options *opt, void *stream, f3m_plan_t **plan_out);

/*
 * f3m_kmvm - y ~= K(X,X) b with the plan's partition (Appendix E, Algorithm 1):
 * per depth the far-field product L_X^T (K (L_Y b)) of Sec. 3 "Interpolating
 * k(x,y)" (P2M, M2L, L2P), then the exact near-field sums of Sec. 3 eq. (1) at
 * the last depth, then the inverse permutation sigma.
 *   b, y   device fp32[n], caller's order; y is overwritten; they must not overlap.
 *   Asynchronous on `stream`: the call only enqueues kernels, it allocates nothing and never waits for
 *   the device (every workspace was sized by f3m_plan); one call in flight per plan (the plan holds the
 *   workspace).  It may therefore be captured into a HIP graph (stream capture on `stream`; the plan's
 *   own second stream joins the capture through an event and is joined back before the call returns):
 *   a replay computes the product of what b holds then, into y.  A captured call records no times
 *   (f3m_stage_times reports the stages of the plan only after it).
 */
f3m_status f3m_kmvm(f3m_plan_t *plan, const float *b, float *y, void *stream);

/*
 * f3m_kmvm_multi - m products with one plan: column j of Y = F3M product of column j of B, the same
 * result as m calls of f3m_kmvm (to rounding: the order of the near-field sums differs).  A solver
 * with several right-hand sides or probe vectors is the intended caller.  Where the near field runs on
 * the 3-D Gram kernel it is evaluated for groups of up to 4 columns at once, which shares its dominant
 * cost, the exponentials; otherwise the call is a loop of single products.
 *   B   device fp32, column j at B + j*ldb, one entry per source (ldb >= number of sources)
 *   Y   device fp32, column j at Y + j*ldy, n entries each (ldy >= n); overwritten; B and Y must not overlap
 *   m   >= 0
 * The first call on a plan allocates work space for 4 columns (about 8 floats per point), kept by the plan.
 * Asynchronous on `stream` after that.
 */
f3m_status f3m_kmvm_multi(f3m_plan_t *plan, const float *B, int64_t ldb, float *Y, int64_t ldy, int m,
                          void *stream);

/*
 * f3m_plan_xy - the plan for v = K(X, Y) b with two point sets: X (nx targets, rows of v) and
 * Y (ny sources, one weight b_j per row), the general form the method is stated in (Sec. 3;
 * Algorithm 1 keeps one treecode per set).
 *   - Both sets get a cube of the same edge E = the largest extent of either set (enclosing
 *     formula of Sec. 3), each anchored at its own per-dimension minimum (the alpha of the
 *     box-index formula of Sec. 4.2), and each is divided on its own grid; the grids have equal
 *     box edges at every depth and are shifted against each other by alpha^Y - alpha^X.
 *   - A pair (box of X, box of Y) is far iff the distance of the box centres is >= eta * (box
 *     edge): sum_d ((c'_d - c_d) + u_d)^2 >= eta^2 with c, c' the integer cells of the target and
 *     the source box and u_d = ((alpha^Y_d - alpha^X_d) / E) * 2^depth, evaluated in fp64 with every
 *     operation rounded on its own, d ascending.
 *   - Algorithm 1 divides while interactions remain and the largest box of X AND the largest box
 *     of Y hold more than leaf_max points.
 *   - small field: |box of X| + |box of Y| <= small_field; smooth field and adaptive rule as for
 *     one set (they depend on the common box edge only).
 * Arguments as f3m_plan_ex; Y is device, ny x D row-major fp32, 0 <= ny < 2^31.  f3m_kmvm on such a
 * plan reads b[ny] and writes y[nx]; with ny == 0 it writes zeros.  The interaction lists of
 * f3m_plan_get_list have one row per box of X and hold ranks of boxes of Y; f3m_plan_get_perm,
 * _get_point_keys, _get_boxes and f3m_info describe the partition of X, the *_source_* calls
 * below that of Y.  (The near-field and M2L kernels specialised for one shared grid in 3-D are
 * not used by such a plan.)
 */
f3m_status f3m_plan_xy(const float *X, int64_t nx, const float *Y, int64_t ny, int D, float lengthscale,
                       int interp_nodes, float eta, const f3m_options *opt, void *stream,
                       f3m_plan_t **plan_out);

/*
 * direct_kmvm - the exact product y_i = sum_j k(x_i,x_j) b_j (Sec. 2, KeOps
 * paragraph), O(n^2) time, O(n) memory, fp32 arithmetic.  Asynchronous on `stream`.
 */
f3m_status direct_kmvm(const float *X, int64_t n, int D, float lengthscale,
                       const float *b, float *y, void *stream);

/*
 * direct_kmvm_rows_f64 - the same exact sums in fp64 for m selected rows, the
 * reference the paper measures its relative error against (Sec. 5, first
 * paragraph: a subset of rows against the entire data set in double precision).
 *   rows  device int64[m], each in [0,n);  y64  device double[m].
 */
f3m_status direct_kmvm_rows_f64(const float *X, int64_t n, int D, float lengthscale,
                                const float *b, const int64_t *rows, int64_t m,
                                double *y64, void *stream);

/*
 * direct_kmvm_rows_f64_static - direct_kmvm_rows_f64 for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels, the same slicing of the sources and therefore the same bits in y64, but the partial sums
 * of the slices live in a static device array of the library (32 MiB per device: 256 slices x 16384
 * rows of doubles) instead of an allocation.  The call allocates and frees nothing and does not wait
 * for the device: it only enqueues two kernels on `stream`.
 *   Arguments as direct_kmvm_rows_f64, with m <= 16384; a larger m returns F3M_ERR_UNSUPPORTED and
 *   enqueues nothing.
 *   Every call on a device shares that device's array: two calls that overlap in time on one device
 *   (different streams, or different threads) race on it and give wrong sums; calls on one stream are
 *   ordered and safe.  Nothing needs clearing between calls (every partial sum that is read is
 *   written first by the same call).
 */
f3m_status direct_kmvm_rows_f64_static(const float *X, int64_t n, int D, float lengthscale,
                                       const float *b, const int64_t *rows, int64_t m,
                                       double *y64, void *stream);

/*
 * direct_kmvm_xy / direct_kmvm_xy_rows_f64 - the same exact sums for two point sets,
 * y_i = sum_j k(x_i, y_j) b_j (Sec. 2): X device nx x D, Y device ny x D, b device fp32[ny],
 * y device fp32[nx]; rows device int64[m], each in [0,nx); y64 device double[m].
 */
f3m_status direct_kmvm_xy(const float *X, int64_t nx, const float *Y, int64_t ny, int D, float lengthscale,
                          const float *b, float *y, void *stream);
f3m_status direct_kmvm_xy_rows_f64(const float *X, int64_t nx, const float *Y, int64_t ny, int D,
                                   float lengthscale, const float *b, const int64_t *rows, int64_t m,
                                   double *y64, void *stream);

/*
 * f3m_cg_solve - kernel ridge regression x = (K(X,X) + lambda I)^{-1} b by conjugate gradients, with
 * the plan's F3M product as the matrix-vector product of the solver (Sec. 5 "Kernel Ridge Regression
 * experiment").  Hestenes-Stiefel recurrences from x_0 = 0 in fp32 vectors with fp64 inner products;
 * stops after the first iteration k with |r_k| <= tol |b| or after max_iter iterations.
 *   plan          a one-set plan (f3m_plan / f3m_plan_ex); a two-set plan is refused (not square)
 *   lambda        ridge parameter, finite and >= 0
 *   b, x          device fp32[n]; x is overwritten (no initial guess is read); they must not overlap
 *   max_iter      >= 0;  tol >= 0 (0: run max_iter iterations)
 *   iters_host    receives the number of iterations made (may be NULL)
 *   history_host  max_iter + 1 floats, history[k] = |r_k| / |b| from the recurrence, k = 0..iterations
 *                 (may be NULL)
 * Allocates four work vectors of n floats for the duration of the call, runs on `stream` and
 * returns when the solve has finished.  F3M_ERR_BREAKDOWN if a search direction p has
 * p.(K + lambda I)p <= 0 (the approximate operator need not be positive definite for tiny lambda).
 */
f3m_status f3m_cg_solve(f3m_plan_t *plan, float lambda, const float *b, float *x, int max_iter, float tol,
                        int *iters_host, float *history_host, void *stream);

/* Destroys the plan (NULL is allowed); waits for the device first.  Its device buffers go back to the
 * library's memory pool, where the next plan finds them again (building plan after plan then costs no
 * hipMalloc / hipFree); the pool keeps at most 96 GiB and gives the rest back to the device at once. */
void f3m_destroy(f3m_plan_t *plan);

/* Gives every cached block of the pool back to the device (hipFree) and returns the bytes freed.  Buffers
 * of living plans are not touched.  Call it when the device memory is wanted for something else. */
int64_t f3m_trim_memory(void);

/* Message of the last failing call on this thread ("" if none). */
const char *f3m_last_error(void);

/* ---- introspection: for parity checks and reports; all outputs are HOST buffers ---- */

/* Fills *out.  The point-pair counts (near_point_pairs, far_point_pairs) are not needed by the
 * product, so the first call on a plan computes them on the device, re-reading every
 * interaction list, and waits for that; later calls only copy.  Not thread-safe on one plan. */
f3m_status f3m_plan_info(const f3m_plan_t *plan, f3m_info *out);

/* perm[k] = caller's index of the k-th point in box order (n entries): the
 * permutation pi of Sec. 4.1; ascending (key, index). */
f3m_status f3m_plan_get_perm(const f3m_plan_t *plan, uint32_t *perm_host);

/* keys of the points at the quantisation depth, in box order (n entries) */
f3m_status f3m_plan_get_point_keys(const f3m_plan_t *plan, uint32_t *keys_host);

/* occupied boxes of a depth: keys[nboxes] ascending, starts[nboxes+1] = index
 * intervals into the box-ordered points (Sec. 4.1 "Box-to-threadblock alignment") */
f3m_status f3m_plan_get_boxes(const f3m_plan_t *plan, int level, uint32_t *keys_host,
                              uint32_t *starts_host);

/* interaction list of a depth as CSR by target box rank; kind 0 = near, 1 = far,
 * 2 = small field (pairs summed directly at that depth, f3m_options.small_field);
 * row_ptr[nboxes+1], cols[pairs] ascending inside a row.  Near lists exist for
 * every depth 0..L, far and small-field lists for 1..L (empty rows at depth 0 and
 * when the rule is off). */
f3m_status f3m_plan_get_list(const f3m_plan_t *plan, int level, int kind,
                             uint64_t *row_ptr_host, uint32_t *cols_host);

/* The source side of a plan (the partition of Y for f3m_plan_xy; for a one-set plan the same
 * partition as the targets'): counts, anchor, and the analogues of f3m_plan_get_perm (ny entries)
 * and f3m_plan_get_boxes. */
typedef struct {
    int64_t n;                                 /* sources */
    int32_t two_sets;                          /* 1 for a plan made by f3m_plan_xy */
    float alpha[F3M_MAX_DIM];                  /* per-dimension minimum of the sources (their cube anchor) */
    int64_t nboxes[F3M_MAX_LEVELS + 1];        /* occupied source boxes per depth 0..L */
    int64_t max_box[F3M_MAX_LEVELS + 1];       /* largest source box per depth */
} f3m_source_info;
f3m_status f3m_plan_source_info(const f3m_plan_t *plan, f3m_source_info *out);
f3m_status f3m_plan_get_source_perm(const f3m_plan_t *plan, uint32_t *perm_host);
f3m_status f3m_plan_get_source_boxes(const f3m_plan_t *plan, int level, uint32_t *keys_host,
                                     uint32_t *starts_host);

/* Stage times of the last plan build and the last f3m_kmvm (synchronises). */
f3m_status f3m_stage_times(f3m_plan_t *plan, f3m_times *out);

/* Far-field kernel times of one depth in the last f3m_kmvm, measured with HIP events on
 * the stream the kernels were launched on: ms_host[0..2] = P2M, M2L, L2P of that depth
 * (zeros if the depth has no far pairs).  Synchronises. */
f3m_status f3m_level_times(f3m_plan_t *plan, int level, float *ms_host);

#ifdef __cplusplus
}
#endif
#endif /* F3M_H */
