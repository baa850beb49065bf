// extern "C" boundary of libf3m: argument checks, error translation, introspection.
#include <cmath>
#include <cstring>
#include <new>

#include "plan.h"

namespace {

thread_local std::string g_last_error;

f3m_status set_error(f3m_status st, const std::string &msg) {
    g_last_error = msg;
    return st;
}

template <class F>
f3m_status guarded(F &&f) {
    try {
        f();
        return F3M_OK;
    } catch (const f3m::Error &e) {
        return set_error(e.status, e.msg);
    } catch (const std::bad_alloc &) {
        return set_error(F3M_ERR_OOM, "host allocation failed");
    } catch (const std::exception &e) {
        return set_error(F3M_ERR_HIP, e.what());
    } catch (...) {
        return set_error(F3M_ERR_HIP, "unknown failure");
    }
}

bool finite_pos(float v) { return std::isfinite(v) && v > 0.f; }

f3m_status check_problem(const float *X, int64_t n, int D, float lengthscale) {
    if (n < 0) return set_error(F3M_ERR_INVALID_ARG, "n must be >= 0");
    if (D < 1 || D > F3M_MAX_DIM) return set_error(F3M_ERR_INVALID_ARG, "D must be in [1,7]");
    if (!finite_pos(lengthscale)) return set_error(F3M_ERR_INVALID_ARG, "lengthscale must be finite and > 0");
    if (n > 0 && !X) return set_error(F3M_ERR_INVALID_ARG, "X is null");
    if (n >= ((int64_t)1 << 31)) return set_error(F3M_ERR_UNSUPPORTED, "n must be below 2^31");
    return F3M_OK;
}

// false for a plan with no targets or no sources: it holds no tables
bool built(const f3m_plan_t *plan) { return plan->n > 0 && plan->ns() > 0; }

template <class T>
void copy_to_host(T *dst, const T *src, size_t count) {
    if (count == 0) return;
    F3M_HIP(hipMemcpy(dst, src, count * sizeof(T), hipMemcpyDeviceToHost));
}

}  // namespace

extern "C" const char *f3m_last_error(void) { return g_last_error.c_str(); }

// plan for one point set (Y == nullptr) or for targets X and sources Y
static f3m_status make_plan(const float *X, int64_t n, const float *Y, int64_t ny, bool two_sets, int D,
                            float lengthscale, int interp_nodes, float eta, const f3m_options *opt, void *stream,
                            f3m_plan_t **plan_out) {
    if (!plan_out) return set_error(F3M_ERR_INVALID_ARG, "plan_out is null");
    *plan_out = nullptr;
    f3m_status st = check_problem(X, n, D, lengthscale);
    if (st != F3M_OK) return st;
    if (two_sets) {
        if (ny < 0) return set_error(F3M_ERR_INVALID_ARG, "ny must be >= 0");
        if (ny > 0 && !Y) return set_error(F3M_ERR_INVALID_ARG, "Y is null");
        if (ny >= ((int64_t)1 << 31)) return set_error(F3M_ERR_UNSUPPORTED, "ny must be below 2^31");
    }
    if (interp_nodes < 2) return set_error(F3M_ERR_INVALID_ARG, "interp_nodes must be >= 2");
    if (!finite_pos(eta)) return set_error(F3M_ERR_INVALID_ARG, "eta (far-field distance ratio) must be finite and > 0");
    if (opt && (opt->leaf_max < 0 || opt->max_depth < 0))
        return set_error(F3M_ERR_INVALID_ARG, "negative option value");
    if (opt && opt->small_field < 0) return set_error(F3M_ERR_INVALID_ARG, "small_field must be >= 0");
    if (opt && opt->route_min_points < 0) return set_error(F3M_ERR_INVALID_ARG, "route_min_points must be >= 0");
    if (opt && !(std::isfinite(opt->eta_smooth) && opt->eta_smooth >= 0.f))
        return set_error(F3M_ERR_INVALID_ARG, "eta_smooth must be finite and >= 0");
    if (interp_nodes > 8) return set_error(F3M_ERR_UNSUPPORTED, "interp_nodes above 8 is not supported");
    double r = std::pow((double)interp_nodes, (double)D);
    if (r > (double)f3m::MAX_NODES) return set_error(F3M_ERR_UNSUPPORTED, "interp_nodes^D exceeds the node cap of 4096");
    if ((double)eta > 1.0e4) return set_error(F3M_ERR_INVALID_ARG, "eta is unreasonably large");

    f3m_plan_s *P = nullptr;
    st = guarded([&] {
        P = new f3m_plan_s();
        P->n = n;
        P->D = D;
        P->p = interp_nodes;
        P->r = (int)std::lround(r);
        P->gamma = lengthscale;
        P->theta = eta;
        P->T = (int)std::ceil((double)eta * (double)eta);
        P->Lq = f3m::quant_depth(D);
        P->leaf_max = (opt && opt->leaf_max > 0) ? opt->leaf_max : 128;
        P->max_depth = opt ? opt->max_depth : 0;
        P->force_all_near = opt ? (opt->force_all_near != 0) : 0;
        P->no_overlap = opt ? (opt->overlap == 0) : 1;
        P->eta_smooth = opt ? opt->eta_smooth : 0.f;
        P->adaptive_far = opt ? (opt->adaptive_far != 0) : 0;
        P->rho = opt ? opt->small_field : 0;
        P->route_min_n = (opt && opt->route_min_points > 0) ? opt->route_min_points : ((int64_t)1 << 24);
        F3M_HIP(hipGetDevice(&P->device));
        if (two_sets) {
            P->src.reset(new f3m_source());
            P->src->n = ny;
        }
        // with no targets there is nothing to compute, with no sources the product is zero
        if (n > 0 && (!two_sets || ny > 0)) f3m::build_plan(*P, X, two_sets ? Y : nullptr, (hipStream_t)stream);
    });
    if (st != F3M_OK) {
        delete P;
        (void)hipGetLastError();
        return st;
    }
    *plan_out = P;
    return F3M_OK;
}

extern "C" {

f3m_status f3m_plan_ex(const float *X, int64_t n, int D, float lengthscale, int interp_nodes, float eta,
                       const f3m_options *opt, void *stream, f3m_plan_t **plan_out) {
    return make_plan(X, n, nullptr, 0, false, D, lengthscale, interp_nodes, eta, opt, stream, plan_out);
}

f3m_status f3m_plan_xy(const float *X, int64_t nx, const float *Y, int64_t ny, int D, float lengthscale,
                       int interp_nodes, float eta, const f3m_options *opt, void *stream, f3m_plan_t **plan_out) {
    return make_plan(X, nx, Y, ny, true, D, lengthscale, interp_nodes, eta, opt, stream, plan_out);
}

f3m_status f3m_plan(const float *X, int64_t n, int D, float lengthscale, int interp_nodes, float eta, void *stream,
                    f3m_plan_t **plan_out) {
    return f3m_plan_ex(X, n, D, lengthscale, interp_nodes, eta, nullptr, stream, plan_out);
}

f3m_status f3m_kmvm(f3m_plan_t *plan, const float *b, float *y, void *stream) {
    if (!plan) return set_error(F3M_ERR_INVALID_ARG, "plan is null");
    if (plan->n == 0) return F3M_OK;
    if (!y) return set_error(F3M_ERR_INVALID_ARG, "y is null");
    if (plan->ns() == 0) return guarded([&] { f3m::run_zero(y, plan->n, (hipStream_t)stream); });   // no sources
    if (!b) return set_error(F3M_ERR_INVALID_ARG, "b is null");
    if (b == y) return set_error(F3M_ERR_INVALID_ARG, "b and y must not overlap");
    return guarded([&] { f3m::run_kmvm(*plan, b, y, (hipStream_t)stream); });
}

f3m_status f3m_kmvm_multi(f3m_plan_t *plan, const float *B, int64_t ldb, float *Y, int64_t ldy, int m, void *stream) {
    if (!plan) return set_error(F3M_ERR_INVALID_ARG, "plan is null");
    if (m < 0) return set_error(F3M_ERR_INVALID_ARG, "m must be >= 0");
    if (m == 0 || plan->n == 0) return F3M_OK;
    if (!Y) return set_error(F3M_ERR_INVALID_ARG, "Y is null");
    if (ldy < plan->n) return set_error(F3M_ERR_INVALID_ARG, "ldy must be at least the number of targets");
    if (plan->ns() == 0)
        return guarded([&] { for (int j = 0; j < m; ++j) f3m::run_zero(Y + (int64_t)j * ldy, plan->n, (hipStream_t)stream); });
    if (!B) return set_error(F3M_ERR_INVALID_ARG, "B is null");
    if (ldb < plan->ns()) return set_error(F3M_ERR_INVALID_ARG, "ldb must be at least the number of sources");
    if (B == Y) return set_error(F3M_ERR_INVALID_ARG, "B and Y must not overlap");
    return guarded([&] { f3m::run_kmvm_multi(*plan, B, ldb, Y, ldy, m, (hipStream_t)stream); });
}

f3m_status direct_kmvm(const float *X, int64_t n, int D, float lengthscale, const float *b, float *y, void *stream) {
    f3m_status st = check_problem(X, n, D, lengthscale);
    if (st != F3M_OK) return st;
    if (n == 0) return F3M_OK;
    if (!b || !y) return set_error(F3M_ERR_INVALID_ARG, "b or y is null");
    if (b == y) return set_error(F3M_ERR_INVALID_ARG, "b and y must not overlap");
    return guarded([&] { f3m::run_direct(X, n, X, n, D, lengthscale, b, y, (hipStream_t)stream); });
}

f3m_status direct_kmvm_xy(const float *X, int64_t nx, const float *Y, int64_t ny, int D, float lengthscale,
                          const float *b, float *y, void *stream) {
    f3m_status st = check_problem(X, nx, D, lengthscale);
    if (st != F3M_OK) return st;
    st = check_problem(Y, ny, D, lengthscale);
    if (st != F3M_OK) return st;
    if (nx == 0) return F3M_OK;
    if (!y) return set_error(F3M_ERR_INVALID_ARG, "y is null");
    if (ny == 0) return guarded([&] { f3m::run_zero(y, nx, (hipStream_t)stream); });
    if (!b) return set_error(F3M_ERR_INVALID_ARG, "b is null");
    if (b == y) return set_error(F3M_ERR_INVALID_ARG, "b and y must not overlap");
    return guarded([&] { f3m::run_direct(X, nx, Y, ny, D, lengthscale, b, y, (hipStream_t)stream); });
}

f3m_status direct_kmvm_rows_f64(const float *X, int64_t n, int D, float lengthscale, const float *b,
                                const int64_t *rows, int64_t m, double *y64, void *stream) {
    f3m_status st = check_problem(X, n, D, lengthscale);
    if (st != F3M_OK) return st;
    if (m < 0) return set_error(F3M_ERR_INVALID_ARG, "m must be >= 0");
    if (m == 0) return F3M_OK;
    if (n == 0) return set_error(F3M_ERR_INVALID_ARG, "rows requested of an empty problem");
    if (!b || !rows || !y64) return set_error(F3M_ERR_INVALID_ARG, "b, rows or y64 is null");
    return guarded([&] { f3m::run_direct_rows_f64(X, X, n, D, lengthscale, b, rows, m, y64, (hipStream_t)stream); });
}

f3m_status direct_kmvm_rows_f64_static(const float *X, int64_t n, int D, float lengthscale, const float *b,
                                       const int64_t *rows, int64_t m, double *y64, void *stream) {
    f3m_status st = check_problem(X, n, D, lengthscale);
    if (st != F3M_OK) return st;
    if (m < 0) return set_error(F3M_ERR_INVALID_ARG, "m must be >= 0");
    if (m == 0) return F3M_OK;
    if (n == 0) return set_error(F3M_ERR_INVALID_ARG, "rows requested of an empty problem");
    if (!b || !rows || !y64) return set_error(F3M_ERR_INVALID_ARG, "b, rows or y64 is null");
    return guarded([&] { f3m::run_direct_rows_f64_static(X, n, D, lengthscale, b, rows, m, y64, (hipStream_t)stream); });
}

f3m_status direct_kmvm_xy_rows_f64(const float *X, int64_t nx, const float *Y, int64_t ny, int D, float lengthscale,
                                   const float *b, const int64_t *rows, int64_t m, double *y64, void *stream) {
    f3m_status st = check_problem(X, nx, D, lengthscale);
    if (st != F3M_OK) return st;
    st = check_problem(Y, ny, D, lengthscale);
    if (st != F3M_OK) return st;
    if (m < 0) return set_error(F3M_ERR_INVALID_ARG, "m must be >= 0");
    if (m == 0) return F3M_OK;
    if (nx == 0) return set_error(F3M_ERR_INVALID_ARG, "rows requested of an empty set of targets");
    if (!rows || !y64) return set_error(F3M_ERR_INVALID_ARG, "rows or y64 is null");
    if (ny == 0) return guarded([&] { F3M_HIP(hipMemsetAsync(y64, 0, sizeof(double) * (size_t)m, (hipStream_t)stream)); });
    if (!b) return set_error(F3M_ERR_INVALID_ARG, "b is null");
    return guarded([&] { f3m::run_direct_rows_f64(X, Y, ny, D, lengthscale, b, rows, m, y64, (hipStream_t)stream); });
}

f3m_status f3m_cg_solve(f3m_plan_t *plan, float lambda, const float *b, float *x, int max_iter, float tol,
                        int *iters_host, float *history_host, void *stream) {
    if (iters_host) *iters_host = 0;
    if (!plan) return set_error(F3M_ERR_INVALID_ARG, "plan is null");
    if (plan->src) return set_error(F3M_ERR_INVALID_ARG, "f3m_cg_solve needs a one-set plan (a square operator)");
    if (!(std::isfinite(lambda) && lambda >= 0.f)) return set_error(F3M_ERR_INVALID_ARG, "lambda must be finite and >= 0");
    if (max_iter < 0) return set_error(F3M_ERR_INVALID_ARG, "max_iter must be >= 0");
    if (!(std::isfinite(tol) && tol >= 0.f)) return set_error(F3M_ERR_INVALID_ARG, "tol must be finite and >= 0");
    if (plan->n == 0) return F3M_OK;
    if (!b || !x) return set_error(F3M_ERR_INVALID_ARG, "b or x is null");
    if (b == x) return set_error(F3M_ERR_INVALID_ARG, "b and x must not overlap");
    return guarded([&] { f3m::run_cg(*plan, lambda, b, x, max_iter, tol, iters_host, history_host, (hipStream_t)stream); });
}

int64_t f3m_trim_memory(void) {
    int64_t freed = 0;
    (void)guarded([&] { freed = (int64_t)f3m::pool_trim(); });
    return freed;
}

void f3m_destroy(f3m_plan_t *plan) {
    if (!plan) return;
    (void)hipDeviceSynchronize();
    delete plan;
}

f3m_status f3m_plan_info(const f3m_plan_t *plan, f3m_info *out) {
    if (!plan || !out) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    if (plan->n > 0 && plan->ns() > 0 && !plan->have_far_point_pairs) {
        // cached on first use; the plan is logically unchanged
        f3m_status st = guarded([&] { f3m::compute_far_point_pairs(*const_cast<f3m_plan_t *>(plan)); });
        if (st != F3M_OK) return st;
    }
    std::memset(out, 0, sizeof(*out));
    out->n = plan->n;
    out->D = plan->D;
    out->interp_nodes = plan->p;
    out->nodes_per_box = plan->r;
    out->depth = plan->L;
    out->quant_depth = plan->Lq;
    out->far_threshold = plan->T;
    out->edge = plan->E;
    out->scale = plan->scale;
    for (int d = 0; d < F3M_MAX_DIM; ++d) out->alpha[d] = plan->alpha[d];
    for (int l = 0; l <= plan->L && built(plan); ++l) {
        out->nboxes[l] = plan->lev[l].nb;
        out->max_box[l] = plan->lev[l].max_box;
        out->near_pairs[l] = plan->lev[l].near_sz;
        out->far_pairs[l] = plan->lev[l].far_sz;
    }
    for (int l = 0; l <= plan->L && built(plan); ++l) out->far_point_pairs[l] = plan->lev[l].far_point_pairs;
    out->near_point_pairs = plan->near_point_pairs;
    out->smooth_depth = plan->smooth_depth;
    for (int l = 0; l <= plan->L && built(plan); ++l) {
        out->small_pairs[l] = plan->lev[l].small_sz;
        out->small_point_pairs[l] = plan->lev[l].small_point_pairs;
    }
    for (int l = 0; l <= F3M_MAX_LEVELS; ++l) out->level_nodes[l] = (l >= 1 && l <= plan->L) ? plan->lev[l].p : 0;
    out->device_bytes = plan->bytes;
    return F3M_OK;
}

f3m_status f3m_plan_get_perm(const f3m_plan_t *plan, uint32_t *perm_host) {
    if (!plan || !perm_host) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    return guarded([&] { copy_to_host(perm_host, plan->perm.p, built(plan) ? (size_t)plan->n : 0); });
}

f3m_status f3m_plan_get_point_keys(const f3m_plan_t *plan, uint32_t *keys_host) {
    if (!plan || !keys_host) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    return guarded([&] { copy_to_host(keys_host, plan->keys.p, built(plan) ? (size_t)plan->n : 0); });
}

f3m_status f3m_plan_get_boxes(const f3m_plan_t *plan, int level, uint32_t *keys_host, uint32_t *starts_host) {
    if (!plan || !keys_host || !starts_host) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    if (!built(plan) || level < 0 || level > plan->L) return set_error(F3M_ERR_INVALID_ARG, "level out of range");
    return guarded([&] {
        const f3m_level &lv = plan->lev[level];
        copy_to_host(keys_host, lv.key.p, (size_t)lv.nb);
        copy_to_host(starts_host, lv.start.p, (size_t)lv.nb + 1);
    });
}

f3m_status f3m_plan_source_info(const f3m_plan_t *plan, f3m_source_info *out) {
    if (!plan || !out) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    std::memset(out, 0, sizeof(*out));
    out->n = plan->ns();
    out->two_sets = plan->src ? 1 : 0;
    for (int d = 0; d < F3M_MAX_DIM; ++d) out->alpha[d] = plan->salpha()[d];
    for (int l = 0; l <= plan->L && built(plan); ++l) {
        out->nboxes[l] = plan->slev(l).nb;
        out->max_box[l] = plan->slev(l).max_box;
    }
    return F3M_OK;
}

f3m_status f3m_plan_get_source_perm(const f3m_plan_t *plan, uint32_t *perm_host) {
    if (!plan || !perm_host) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    return guarded([&] { copy_to_host(perm_host, plan->sperm(), built(plan) ? (size_t)plan->ns() : 0); });
}

f3m_status f3m_plan_get_source_boxes(const f3m_plan_t *plan, int level, uint32_t *keys_host, uint32_t *starts_host) {
    if (!plan || !keys_host || !starts_host) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    if (!built(plan) || level < 0 || level > plan->L) return set_error(F3M_ERR_INVALID_ARG, "level out of range");
    return guarded([&] {
        const f3m_level &lv = plan->slev(level);
        copy_to_host(keys_host, lv.key.p, (size_t)lv.nb);
        copy_to_host(starts_host, lv.start.p, (size_t)lv.nb + 1);
    });
}

f3m_status f3m_plan_get_list(const f3m_plan_t *plan, int level, int kind, uint64_t *row_ptr_host, uint32_t *cols_host) {
    if (!plan || !row_ptr_host || !cols_host) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    if (!built(plan) || level < 0 || level > plan->L) return set_error(F3M_ERR_INVALID_ARG, "level out of range");
    if (kind < 0 || kind > 2) return set_error(F3M_ERR_INVALID_ARG, "kind must be 0 (near), 1 (far) or 2 (small field)");
    return guarded([&] {
        const f3m_level &lv = plan->lev[level];
        if (kind == 2) {
            if (lv.small_ptr.p) {
                copy_to_host(row_ptr_host, lv.small_ptr.p, (size_t)lv.nb + 1);
                copy_to_host(cols_host, lv.small_col.p, (size_t)lv.small_sz);
            } else {
                std::memset(row_ptr_host, 0, sizeof(uint64_t) * ((size_t)lv.nb + 1));
            }
            return;
        }
        copy_to_host(row_ptr_host, kind ? lv.far_ptr.p : lv.near_ptr.p, (size_t)lv.nb + 1);
        if (kind && lv.far_implicit) {
            // this depth keeps only the lengths of its far rows
            f3m::DevBuf<uint32_t> cols;
            cols.alloc((size_t)lv.far_sz);
            f3m::materialize_far(*plan, level, cols.p, nullptr);
            copy_to_host(cols_host, cols.p, (size_t)lv.far_sz);
        } else {
            copy_to_host(cols_host, kind ? lv.far_col.p : lv.near_col.p, (size_t)(kind ? lv.far_sz : lv.near_sz));
        }
    });
}

f3m_status f3m_stage_times(f3m_plan_t *plan, f3m_times *out) {
    if (!plan || !out) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    return guarded([&] {
        f3m_times t = plan->times;
        if (plan->have_kmvm_times) {
            F3M_HIP(hipEventSynchronize(plan->ev[12]));
            F3M_HIP(hipEventElapsedTime(&t.permute_in, plan->ev[8], plan->ev[9]));
            F3M_HIP(hipEventSynchronize(plan->ev_p2p1));
            F3M_HIP(hipEventElapsedTime(&t.p2p, plan->ev_p2p0, plan->ev_p2p1));
            F3M_HIP(hipEventElapsedTime(&t.permute_out, plan->ev[11], plan->ev[12]));
            F3M_HIP(hipEventElapsedTime(&t.kmvm_total, plan->ev[8], plan->ev[12]));
            t.p2m = t.m2l = t.l2p = 0.f;
            for (int l = 1; l <= plan->L; ++l) {
                if (plan->lev[l].far_sz == 0 || plan->far_events.size() < (size_t)(l + 1) * 6) continue;
                hipEvent_t *ev = &plan->far_events[(size_t)l * 6];
                if (!ev[5]) continue;
                float ms = 0.f;
                F3M_HIP(hipEventElapsedTime(&ms, ev[0], ev[1])); t.p2m += ms;
                F3M_HIP(hipEventElapsedTime(&ms, ev[2], ev[3])); t.m2l += ms;
                F3M_HIP(hipEventElapsedTime(&ms, ev[4], ev[5])); t.l2p += ms;
            }
        }
        *out = t;
    });
}

f3m_status f3m_level_times(f3m_plan_t *plan, int level, float *ms_host) {
    if (!plan || !ms_host) return set_error(F3M_ERR_INVALID_ARG, "null argument");
    if (!built(plan) || level < 0 || level > plan->L) return set_error(F3M_ERR_INVALID_ARG, "level out of range");
    return guarded([&] {
        ms_host[0] = ms_host[1] = ms_host[2] = 0.f;
        if (!plan->have_kmvm_times || plan->lev[level].far_sz == 0 || plan->far_events.size() < (size_t)(level + 1) * 6)
            return;
        hipEvent_t *ev = &plan->far_events[(size_t)level * 6];
        if (!ev[5]) return;
        F3M_HIP(hipEventSynchronize(plan->ev[12]));
        for (int k = 0; k < 3; ++k) F3M_HIP(hipEventElapsedTime(&ms_host[k], ev[2 * k], ev[2 * k + 1]));
    });
}

}  // extern "C"
