// f3m_cg_solve: kernel ridge regression, alpha = (k(X,X) + lambda I)^{-1} b, by conjugate gradients with
// the F3M product as the solver's matrix-vector product (arXiv 2202.01085, Sec. 5 "Kernel Ridge
// Regression experiment"; the paper plugs F3M into a conjugate-gradient solver the same way).
// Textbook Hestenes-Stiefel recurrences from x_0 = 0.  Vectors are fp32 in HBM; every inner product
// is accumulated in fp64 in a fixed order (grid-stride partial sums, one block adds the partials),
// and the step lengths stay in device memory, so an iteration costs one f3m_kmvm, three fused
// vector passes (48 n bytes) and one 40-byte copy to the host for the stopping test.
// The solve works in the plan's box order: b is permuted once on the way in and x once on the
// way out (inner products do not depend on the order), so the products inside the loop skip
// both permutations of f3m_kmvm.
#include <cmath>
#include <vector>

#include "plan.h"

namespace f3m {

constexpr int CG_NT = 256;
constexpr int CG_BLOCKS = 2048;

// scalars of the recurrence in device memory
enum { S_RS = 0, S_PQ = 1, S_ALPHA = 2, S_RS_NEW = 3, S_BETA = 4, S_COUNT = 5 };

__device__ inline void block_sum_to(double v, double *dst) {
    __shared__ double sm[CG_NT / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int k = 0; k < CG_NT / 64; ++k) s += sm[k];
        *dst = s;
    }
}

// box order: x = 0, r = p = b[perm]; partial sums of b . b
__global__ __launch_bounds__(CG_NT) void cg_init_kernel(const float *__restrict__ b, const uint32_t *__restrict__ perm,
                                                        float *__restrict__ x, float *__restrict__ r,
                                                        float *__restrict__ p, int64_t n, double *__restrict__ part) {
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * CG_NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * CG_NT) {
        const float v = b[perm[i]];
        x[i] = 0.f;
        r[i] = v;
        p[i] = v;
        s += (double)v * (double)v;
    }
    block_sum_to(s, part + blockIdx.x);
}

// q = K p on entry; q <- q + lambda p; partial sums of p . q
__global__ __launch_bounds__(CG_NT) void cg_shift_dot_kernel(const float *__restrict__ p, float *__restrict__ q,
                                                             float lambda, int64_t n, double *__restrict__ part) {
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * CG_NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * CG_NT) {
        const float pv = p[i];
        const float qv = fmaf(lambda, pv, q[i]);
        q[i] = qv;
        s += (double)pv * (double)qv;
    }
    block_sum_to(s, part + blockIdx.x);
}

// x += alpha p, r -= alpha q; partial sums of r . r
__global__ __launch_bounds__(CG_NT) void cg_update_kernel(float *__restrict__ x, float *__restrict__ r,
                                                          const float *__restrict__ p, const float *__restrict__ q,
                                                          const double *__restrict__ scal, int64_t n,
                                                          double *__restrict__ part) {
    const float alpha = (float)scal[S_ALPHA];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * CG_NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * CG_NT) {
        x[i] = fmaf(alpha, p[i], x[i]);
        const float rv = fmaf(-alpha, q[i], r[i]);
        r[i] = rv;
        s += (double)rv * (double)rv;
    }
    block_sum_to(s, part + blockIdx.x);
}

// p = r + beta p
__global__ __launch_bounds__(CG_NT) void cg_direction_kernel(float *__restrict__ p, const float *__restrict__ r,
                                                             const double *__restrict__ scal, int64_t n) {
    const float beta = (float)scal[S_BETA];
    for (int64_t i = (int64_t)blockIdx.x * CG_NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * CG_NT)
        p[i] = fmaf(beta, p[i], r[i]);
}

// the solution back in the caller's order
__global__ __launch_bounds__(CG_NT) void cg_unpermute_kernel(const float *__restrict__ xs,
                                                             const uint32_t *__restrict__ perm, int64_t n,
                                                             float *__restrict__ x) {
    for (int64_t i = (int64_t)blockIdx.x * CG_NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * CG_NT)
        x[perm[i]] = xs[i];
}

// adds the partial sums in ascending order and advances the scalars:
//   mode 0: rs = sum                      (after cg_init_kernel)
//   mode 1: pq = sum, alpha = rs / pq     (after cg_shift_dot_kernel)
//   mode 2: rs_new = sum, beta = rs_new / rs, rs = rs_new   (after cg_update_kernel)
__global__ __launch_bounds__(CG_NT) void cg_reduce_kernel(const double *__restrict__ part, int nparts,
                                                          double *__restrict__ scal, int mode) {
    __shared__ double total;
    double s = 0.0;
    for (int k = threadIdx.x; k < nparts; k += CG_NT) s += part[k];
    block_sum_to(s, &total);
    __syncthreads();
    if (threadIdx.x == 0) {
        const double sum = total;
        if (mode == 0) {
            scal[S_RS] = sum;
        } else if (mode == 1) {
            scal[S_PQ] = sum;
            scal[S_ALPHA] = scal[S_RS] / sum;
        } else {
            scal[S_RS_NEW] = sum;
            scal[S_BETA] = sum / scal[S_RS];
            scal[S_RS] = sum;
        }
    }
}

void run_cg(f3m_plan_s &P, float lambda, const float *b, float *x, int max_iter, float tol, int *iters_host,
            float *history_host, hipStream_t st) {
    const int64_t n = P.n;
    DevBuf<float> xs, r, p, q;   // box order
    DevBuf<double> part, scal;
    xs.alloc((size_t)n);
    r.alloc((size_t)n);
    p.alloc((size_t)n);
    q.alloc((size_t)n);
    const int blocks = (int)std::min<int64_t>(CG_BLOCKS, cdiv(n, CG_NT));
    part.alloc((size_t)blocks);
    scal.alloc(S_COUNT);
    F3M_HIP(hipMemsetAsync(scal.p, 0, S_COUNT * sizeof(double), st));
    double h[S_COUNT];
    auto fetch = [&] {
        F3M_HIP(hipMemcpyAsync(h, scal.p, sizeof(h), hipMemcpyDeviceToHost, st));
        F3M_HIP(hipStreamSynchronize(st));
    };
    cg_init_kernel<<<dim3(blocks), dim3(CG_NT), 0, st>>>(b, P.perm.p, xs.p, r.p, p.p, n, part.p);
    cg_reduce_kernel<<<dim3(1), dim3(CG_NT), 0, st>>>(part.p, blocks, scal.p, 0);
    F3M_HIP(hipGetLastError());
    fetch();
    const double nb = std::sqrt(h[S_RS]);
    int it = 0;
    if (history_host) history_host[0] = nb > 0.0 ? 1.f : 0.f;
    if (!std::isfinite(nb)) fail(F3M_ERR_NONFINITE, "the right-hand side holds a NaN or an infinity");
    while (nb > 0.0 && it < max_iter) {
        run_kmvm(P, p.p, q.p, st, true);
        cg_shift_dot_kernel<<<dim3(blocks), dim3(CG_NT), 0, st>>>(p.p, q.p, lambda, n, part.p);
        cg_reduce_kernel<<<dim3(1), dim3(CG_NT), 0, st>>>(part.p, blocks, scal.p, 1);
        cg_update_kernel<<<dim3(blocks), dim3(CG_NT), 0, st>>>(xs.p, r.p, p.p, q.p, scal.p, n, part.p);
        cg_reduce_kernel<<<dim3(1), dim3(CG_NT), 0, st>>>(part.p, blocks, scal.p, 2);
        F3M_HIP(hipGetLastError());
        fetch();
        ++it;
        if (!(h[S_PQ] > 0.0) || !std::isfinite(h[S_RS_NEW])) {
            if (iters_host) *iters_host = it;
            fail(F3M_ERR_BREAKDOWN,
                 "conjugate gradients broke down: p.(K + lambda I)p is not positive (the approximate operator is not "
                 "positive definite along a search direction; raise lambda or the accuracy of the plan)");
        }
        const double res = std::sqrt(h[S_RS_NEW]);
        if (history_host) history_host[it] = (float)(res / nb);
        if (res <= (double)tol * nb) break;
        cg_direction_kernel<<<dim3(blocks), dim3(CG_NT), 0, st>>>(p.p, r.p, scal.p, n);
        F3M_HIP(hipGetLastError());
    }
    if (iters_host) *iters_host = it;
    cg_unpermute_kernel<<<dim3(blocks), dim3(CG_NT), 0, st>>>(xs.p, P.perm.p, n, x);
    F3M_HIP(hipGetLastError());
    F3M_HIP(hipStreamSynchronize(st));   // the work vectors are released on return
}

}  // namespace f3m
