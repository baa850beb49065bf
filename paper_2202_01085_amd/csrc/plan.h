// The plan object: everything of Algorithm 1 that does not depend on b.
#pragma once
#include <memory>

#include "common.h"

struct f3m_level {
    int64_t nb = 0;                     // occupied boxes
    int64_t max_box = 0;
    f3m::DevBuf<uint32_t> key;          // [nb]   box key at this depth, ascending
    f3m::DevBuf<uint32_t> start;        // [nb+1] index interval into the box-ordered points
    f3m::DevBuf<uint32_t> parent;       // [nb]   rank of the parent one depth up
    f3m::DevBuf<uint32_t> cstart;       // [nb+1] rank interval of the children one depth down
    f3m::DevBuf<int32_t> cell;          // [nb*D] integer cell coordinates
    f3m::DevBuf<uint64_t> near_ptr, far_ptr;   // [nb+1]
    f3m::DevBuf<uint32_t> near_col, far_col;
    f3m::DevBuf<uint32_t> far_ord;      // [far_sz] the far rows in the order of the partners' row-major cell index (grouped M2L)
    int64_t near_sz = 0, far_sz = 0;
    int64_t far_point_pairs = 0;        // sum of |p||q| over the far pairs of this depth
    // small field (Sec. 4.2): pairs summed directly at this depth, and the target tiles of their rows
    f3m::DevBuf<uint64_t> small_ptr;    // [nb+1]
    f3m::DevBuf<uint32_t> small_col;
    int64_t small_sz = 0, small_point_pairs = 0;
    int64_t sm_ntiles = 0;
    f3m::DevBuf<uint32_t> sm_tile_box, sm_tile_first;
    // P2M work split: a chunk is a run of at most P2M_CHUNK points of one box
    int64_t nchunks = 0;
    f3m::DevBuf<uint32_t> chunk_box;    // [nchunks]
    f3m::DevBuf<uint32_t> chunk_first;  // [nb+1] first chunk of each box
    // boxes with very many chunks (few, huge boxes): a slice is a run of at most P2M_SLICE chunks of one
    // box, and the partial node weights are added slice by slice first
    int64_t nslices = 0;
    f3m::DevBuf<uint32_t> slice_box, slice_first;
    // D = 3, 4 nodes/dim, far ratio 2: the M2L enumerates the far partners on the candidate grid
    // around the parent (m2l.hip); far_ptr keeps the row lengths, far_col stays empty
    bool far_implicit = false;
    // ... and, without a small field, per box of the depth ABOVE: the rank of the candidate at each of the 216
    // positions of the grid around it and its child of each parity (~0: none)
    f3m::DevBuf<uint32_t> st_cand, st_child;
    // Sec. 4.3: nodes per dimension used at this depth (interp_nodes, 3 under the adaptive rule, or 0 =
    // the far pairs of the depth are dropped), r = p^D, and whether every pair of the depth is interpolated
    int p = 0, r = 0;
    bool smooth = false;
    // 1-D factors of the node-to-node kernel matrix, [2*omax+1][p][p]
    f3m::DevBuf<float> gtab;
    int gtab_omax = 0;
    // node weights / node potentials kept per depth when they are passed between depths
    f3m::DevBuf<float> Wl, Vl;          // [nb*64]
};

// Tables of the three-pass permutation between the caller's order and the box order of one point set
// (route.hip): per pass the place of every value in the LDS copy of its tile, per tile the first place of each
// digit and where the tile's run of each digit lies in the next order.
struct f3m_route {
    int64_t n = 0, ntiles = 0;
    int s2 = 0, B1 = 1, B2 = 1;
    f3m::DevBuf<uint16_t> slot1, slot2, off3;      // [n] each
    f3m::DevBuf<uint32_t> dstart1, dstart2;        // [ntiles][257]
    f3m::DevBuf<uint32_t> gofs1, gofs2;            // [ntiles][256]
};

// The partition of the source set Y of a two-set plan, v = K(X, Y) b (Sec. 3 states the method for
// two data matrices; Algorithm 1 keeps one treecode per set).  Both sets are divided by cubes of
// the same edge, each anchored at its own per-dimension minimum, so the two grids have equal box
// edges at every depth and are shifted against each other.  A one-set plan has no such object.
struct f3m_source {
    int64_t n = 0;
    float alpha[F3M_MAX_DIM] = {0};
    f3m::DevBuf<uint32_t> keys, perm;   // [n]
    f3m::DevBuf<float> Xs;              // [n*D] coordinates in box order, padded
    std::unique_ptr<f3m_route> route;   // large sets: the right-hand side comes into box order in three passes
    f3m_level lev[F3M_MAX_LEVELS + 1];  // box tables and P2M work splits only (no lists)
};

struct f3m_plan_s {
    int64_t n = 0;                              // targets (rows of X); also the sources of a one-set plan
    int D = 0, p = 0, r = 0;
    int Lq = 0, L = 0, T = 4;
    float gamma = 1.f, theta = 2.f;
    float E = 0.f, scale = 0.f;
    float alpha[F3M_MAX_DIM] = {0};
    int leaf_max = 128, max_depth = 0, force_all_near = 0, no_overlap = 0;
    float eta_smooth = 0.f;                     // smooth-field limit of Sec. 4.3 (0 = off)
    int adaptive_far = 0;                       // adaptive far-field node rule of Sec. 4.3
    int64_t rho = 0;                            // small-field limit of Sec. 4.2 (0 = off)
    int smooth_depth = -1;                      // depth whose adjacent pairs are interpolated, or -1
    hipStream_t side = nullptr;                 // second stream for the near field
    hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_p2p0 = nullptr, ev_p2p1 = nullptr;
    int device = 0;
    int64_t bytes = 0;
    int64_t near_point_pairs = 0;

    f3m::DevBuf<uint32_t> keys;   // [n] keys at depth Lq, box order
    f3m::DevBuf<uint32_t> perm;   // [n]
    f3m::DevBuf<float> Xs;        // [n*D] coordinates in box order, row-major
    f3m::DevBuf<float> bs, ys;    // [n] right-hand side / far-field result in box order
    f3m::DevBuf<float> yn;        // [n] near-field result in box order
    f3m::DevBuf<float> multi_bs, multi_yn;   // [4][ns + pad], [4][n]: a group of right-hand sides in box order and its
                                             // near-field results (f3m_kmvm_multi; allocated on first use)
    f3m::DevBuf<float> p2p_part;  // [slices][n] partial near-field sums when target tiles are split (few targets)
    f3m::DevBuf<float> W, V;      // [max_l nb_l * r] node weights / node potentials of one depth
    f3m::DevBuf<float> Wpart;     // [max_l nchunks_l * r] partial node weights
    f3m::DevBuf<double> Wslice;   // [max_l nslices_l * r] sums of the partial node weights of a slice
    // near-field work split: a tile is a run of at most 64 targets of one leaf box (the full runs of 64, and the
    // last run if it is not an overflow tile)
    int64_t ntiles = 0;
    f3m::DevBuf<uint32_t> tile_box, tile_first;   // [ntiles], [nb_L+1]
    // ... and overflow tiles: a last run of a leaf box with so few targets (<= 10, <= 8 above 4-D) that the
    // kernel with the sources on the lanes is cheaper; at most one per box
    int64_t notiles = 0;
    f3m::DevBuf<uint32_t> otile_box, otile_first;
    // ... and pairs of tiles (D = 3, Gram near field, one point set): the first runs of two leaf boxes a, a + 1 with
    // the same parent and cells next to each other are worked by one wavefront, which shares the preparation of
    // the sources near both.  pair_box[i] = a; paired[b] != 0 for both boxes of a pair; rtile_* is the tile list
    // without the first runs of paired boxes (tile_* keeps every run: the products with several right-hand sides
    // and the split near field use it).
    int64_t npairs = 0, nrtiles = 0;
    f3m::DevBuf<uint32_t> pair_box, pair_first;
    f3m::DevBuf<uint8_t> paired;
    f3m::DevBuf<uint32_t> rtile_box, rtile_first;
    f3m_level lev[F3M_MAX_LEVELS + 1];          // boxes of X (targets); lists by target box
    std::unique_ptr<f3m_source> src;            // two-set plan: the partition of Y (sources)
    // the source side of either kind of plan
    const f3m_level &slev(int l) const { return src ? src->lev[l] : lev[l]; }
    f3m_level &slev(int l) { return src ? src->lev[l] : lev[l]; }
    int64_t ns() const { return src ? src->n : n; }
    const float *Ys() const { return src ? src->Xs.p : Xs.p; }
    const uint32_t *sperm() const { return src ? src->perm.p : perm.p; }
    const float *salpha() const { return src ? src->alpha : alpha; }
    // grid shift of a depth in units of its box edge, u_d = ((alpha^Y_d - alpha^X_d) / E) 2^depth: the
    // centre of source cell c' minus the centre of target cell c is ((c' - c) + u) box edges
    void grid_shift(int level, double *u) const {
        for (int d = 0; d < D; ++d) {
            const double diff = (double)salpha()[d] - (double)alpha[d];
            const double q = (src && E > 0.f) ? diff / (double)E : 0.0;
            u[d] = q * (double)(1ull << level);
        }
    }
    int tree_lmin = 0, tree_lmax = 0;   // tree_lmin > 0: node weights/potentials are passed between depths
                                        // tree_lmin..tree_lmax (D = 3, 4 nodes/dim); other depths work
                                        // straight from the points
    f3m::DevBuf<float> transfer;        // [2][4][4] parent basis at the child's nodes
    // large n: both permutations of a product run as three streaming passes (route.hip); the two work
    // vectors hold max(n, sources) floats each
    int64_t route_min_n = 0;                    // the passes are used from this many points on
    std::unique_ptr<f3m_route> route;           // of the targets (and of the sources of a one-set plan)
    f3m::DevBuf<float> route_a, route_b;
    const f3m_route *sroute() const { return src ? src->route.get() : route.get(); }

    hipEvent_t ev[16] = {nullptr};
    std::vector<hipEvent_t> far_events;   // 6 per depth, around the far-field kernels of that depth
    bool have_plan_times = false, have_kmvm_times = false, have_far_point_pairs = false;
    f3m_times times = {};
    ~f3m_plan_s();
};

namespace f3m {

constexpr int P2M_CHUNK = 256;
constexpr int P2M_SLICE = 512;   // chunks per slice of the two-stage sum of partial node weights
// largest last run of a leaf box that is treated as an overflow tile (near field with the sources on the lanes):
// beyond about 10 targets a half-filled 64-wide tile is the cheaper of the two (measured at n = 1e9)
constexpr int overflow_targets(int D) { return D <= 4 ? 10 : 8; }
constexpr int PAD_POINTS = 64;   // zero padding behind Xs and bs
constexpr int MAX_NODES = 4096;

int quant_depth(int D);
bool smooth_rule(double E, int depth, int D, double gamma, double eta_smooth);   // Sec. 4.3 smoothness criterion
int adaptive_nodes(double E, int depth, double gamma, int p);                   // Sec. 4.3 node rule (0: dropped)

// plan.hip
void build_plan(f3m_plan_s &P, const float *X, const float *Y, hipStream_t st);   // Y == nullptr: one set (P.src set otherwise)
void compute_far_point_pairs(f3m_plan_s &P);   // near_point_pairs and lev[].far_point_pairs, once (synchronises)
// route.hip: permutations of large vectors as three streaming passes with tables built once per plan
void route_build(f3m_route &R, const uint32_t *perm, int64_t n, int64_t *tally, hipStream_t st);   // synchronises
void route_scatter(const f3m_route &R, const float *in, const float *in2, float *out, float *tmp_a, float *tmp_b,
                   hipStream_t st);                                   // out[perm[k]] = in[k] (+ in2[k])
void route_gather(const f3m_route &R, const float *in, float *out, float *tmp_a, float *tmp_b, hipStream_t st);
                                                                      // out[k] = in[perm[k]]
void route_gather_rows3(const f3m_route &R, const float *in, float *out, float *tmp, hipStream_t st);
                                                                      // rows of 3 floats; tmp: 3 n floats
void materialize_far(const f3m_plan_s &P, int level, uint32_t *cols_dev, hipStream_t st);   // far rows of an implicit depth
// kmvm.hip
// box_order: b and y are already in the plan's box order (one-set plans only; used by the solver)
void run_kmvm(f3m_plan_s &P, const float *b, float *y, hipStream_t st, bool box_order = false);
void run_kmvm_multi(f3m_plan_s &P, const float *B, int64_t ldb, float *Y, int64_t ldy, int m, hipStream_t st);
int p2p_nsplit(const f3m_plan_s &P, int l, int64_t ntiles);   // source slices per target tile of the near field (1: none)
bool p2p_pairs_allowed(const f3m_plan_s &P);                  // the near field of the last depth may work tiles in pairs
void run_zero(float *y, int64_t n, hipStream_t st);   // y = 0 with a fill kernel
// exact sums of targets X (nx rows) against sources Y (ny rows, weights b); X == Y for one set
void run_direct(const float *X, int64_t nx, const float *Y, int64_t ny, int D, float gamma, const float *b, float *y,
                hipStream_t st);
void run_direct_rows_f64(const float *X, const float *Y, int64_t ny, int D, float gamma, const float *b,
                         const int64_t *rows, int64_t m, double *y64, hipStream_t st);
// the same with the partial sums in a static device array: no allocation, no wait (m <= 16384)
void run_direct_rows_f64_static(const float *X, int64_t n, int D, float gamma, const float *b, const int64_t *rows,
                                int64_t m, double *y64, hipStream_t st);
void upload_transfer(f3m_plan_s &P, hipStream_t st);            // parent-basis-at-child-nodes table
void upload_kron_tables(f3m_plan_s &P, hipStream_t st);         // per-dimension kernel factors of every far depth
void build_far_orders(f3m_plan_s &P, hipStream_t st);           // far rows in row-major cell order for the grouped M2L
// solve.hip: conjugate gradients for (K + lambda I) x = b on a one-set plan (synchronises)
void run_cg(f3m_plan_s &P, float lambda, const float *b, float *x, int max_iter, float tol, int *iters_host,
            float *history_host, hipStream_t st);
// m2l.hip
bool m2l_stencil_applies(const f3m_plan_s &P);
void build_stencil_tables(f3m_plan_s &P, int level, hipStream_t st);
bool stencil_tables_alloc(f3m_plan_s &P, int level, hipStream_t st);   // false: the depth has no such tables   // after the lists of the depth exist                   // D = 3, 4 nodes/dim, far ratio 2
bool run_m2l_stencil(f3m_plan_s &P, int level, const float *W, float *V, hipStream_t st, bool zero_row = false);  // false: does not apply

}  // namespace f3m
