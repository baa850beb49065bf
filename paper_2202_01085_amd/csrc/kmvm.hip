// f3m_kmvm and direct_kmvm: the floating-point passes.
// (arXiv 2202.01085: Sec. 3 eq. (1) near field; Sec. 3 "Interpolating k(x,y)" and Fig. 4
//  for the three far-field passes v1 = L_Y b, v2 = K v1, v = L_X^T v2; Appendix E
//  Algorithm 1 for the order of the passes.)
#include <algorithm>
#include <cmath>

#include <mutex>
#include <type_traits>

#include "plan.h"

// Partial sums of direct_kmvm_rows_f64_static, for callers that may not allocate: up to 256 source
// slices of up to 16384 rows (32 MiB, held on every device the library runs on until the process
// ends).  Host code never uses this name as an address: it asks for the array's address on the
// current device once per device (rows_static_scratch) and passes that pointer to the kernels.
constexpr int ROWS_MAX_SLICES = 256;
constexpr int64_t ROWS_STATIC_MAX_M = 16384;
static __device__ __align__(256) double scratch[(size_t)ROWS_MAX_SLICES * (size_t)ROWS_STATIC_MAX_M];

namespace f3m {

// address of `scratch` on the current device (every device holds its own copy at its own address)
static double *rows_static_scratch() {
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static double *ptr[MAX_DEVICES] = {};
    int dev = 0;
    F3M_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) fail(F3M_ERR_UNSUPPORTED, "device ordinal above 63");
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        double *q = nullptr;
        F3M_HIP(hipGetSymbolAddress((void **)&q, HIP_SYMBOL(scratch)));
        if (!q) fail(F3M_ERR_HIP, "hipGetSymbolAddress gave a null address for the static scratch");
        ptr[dev] = q;
    }
    return ptr[dev];
}

constexpr int P_MAX = 8;  // interpolation nodes per dimension supported by the kernels

// Chebyshev nodes of the second kind s_i = cos(i pi/(p-1)) and the reciprocal denominators
// of the product-form Lagrange basis (Sec. 3 "Lagrange interpolation").
struct NodeArg {
    float s[P_MAX];
    float invden[P_MAX];
};
struct CentreArg {
    double alpha[F3M_MAX_DIM];
    double edge;      // l = E / 2^level
    double inv_half;  // 2 / l
};

// 2-D launch shape for `count` blocks: the runtime limits grid.x * block.x to 32 bits, so
// large block counts are folded over y; kernels recover the index with block_index().
static dim3 grid_for(int64_t count) {
    const int64_t gx = 1 << 16;
    if (count <= gx) return dim3((unsigned)(count > 0 ? count : 1), 1, 1);
    return dim3((unsigned)gx, (unsigned)cdiv(count, gx), 1);
}
__device__ inline int64_t block_index() { return (int64_t)blockIdx.y * gridDim.x + blockIdx.x; }

static NodeArg make_nodes(int p) {
    NodeArg a{};
    double s[P_MAX];
    for (int i = 0; i < p; ++i) s[i] = std::cos((double)i * M_PI / (double)(p - 1));
    for (int i = 0; i < p; ++i) {
        double den = 1.0;
        for (int j = 0; j < p; ++j)
            if (j != i) den *= s[i] - s[j];
        a.s[i] = (float)s[i];
        a.invden[i] = (float)(1.0 / den);
    }
    return a;
}

// box centres of a depth: of the target grid, or of the source grid (its own anchor in a two-set plan)
static CentreArg make_centre(const f3m_plan_s &P, int level, bool source = false) {
    CentreArg c{};
    for (int d = 0; d < P.D; ++d) c.alpha[d] = (double)(source ? P.salpha()[d] : P.alpha[d]);
    c.edge = (double)P.E / std::ldexp(1.0, level);
    c.inv_half = 2.0 / c.edge;
    return c;
}

// ------------------------------------------------------------------------------------
// permutation in and out (the reindexing vector sigma of Sec. 4.2)
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_kernel(const float *__restrict__ b, const uint32_t *__restrict__ perm,
                                                     int64_t n, float *__restrict__ bs) {
    int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) bs[k] = b[perm[k]];
}
// y = far-field part + near-field part, back in the caller's order
__global__ __launch_bounds__(256) void scatter_kernel(const float *__restrict__ ys, const float *__restrict__ yn,
                                                      const uint32_t *__restrict__ perm, int64_t n,
                                                      float *__restrict__ y) {
    int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) y[perm[k]] = ys[k] + yn[k];
}
// the same two steps for a caller that keeps its vectors in box order (the solver)
__global__ __launch_bounds__(256) void copy_kernel(const float *__restrict__ b, int64_t n, float *__restrict__ bs) {
    int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) bs[k] = b[k];
}
__global__ __launch_bounds__(256) void add_kernel(const float *__restrict__ ys, const float *__restrict__ yn, int64_t n,
                                                  float *__restrict__ y) {
    int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) y[k] = ys[k] + yn[k];
}
__global__ __launch_bounds__(256) void zero_kernel(float *__restrict__ p, int64_t n) {
    int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k < n) p[k] = 0.f;
}

// ------------------------------------------------------------------------------------
// near field (Sec. 3 eq. (1)): one wavefront per run of <= 64 targets of a leaf box, one
// lane per target; the sources of the near boxes are wave-uniform, so they arrive through
// the scalar data path and every vector instruction works on 64 distinct pairs.
//   k(x,y) = exp2( nc2 * |x-y|^2 ),  nc2 = -log2(e) / (2 gamma^2)
// All near-field kernels take the targets as (Xt, startT) and the sources as (Xs, bs, start): the
// box-ordered points and point intervals of the target boxes and of the source boxes.  For one
// point set both are the same arrays; for K(X, Y) the columns of a list are ranks of boxes of Y.
// ------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void p2p_kernel(const float *__restrict__ Xt, const uint32_t *__restrict__ startT,
                                                 const float *__restrict__ Xs, const float *__restrict__ bs,
                                                 const uint32_t *__restrict__ start,
                                                 const uint64_t *__restrict__ near_ptr,
                                                 const uint32_t *__restrict__ near_col,
                                                 const uint32_t *__restrict__ tile_box,
                                                 const uint32_t *__restrict__ tile_first, int64_t ntiles,
                                                 float nc2, float *__restrict__ ys, int accumulate) {
    const int64_t t = block_index();
    if (t >= ntiles) return;
    const uint32_t a = tile_box[t];
    const uint32_t k0 = startT[a] + (uint32_t)(t - tile_first[a]) * 64u;
    const uint32_t kend = startT[a + 1];
    const uint32_t k = k0 + threadIdx.x;
    const bool active = k < kend;
    float xi[D];
#pragma unroll
    for (int d = 0; d < D; ++d) xi[d] = active ? Xt[(int64_t)k * D + d] : 0.f;
    double acc = 0.0;   // the runs are added in fp64 (one addition per 32 sources)
    const uint64_t e1 = near_ptr[a + 1];
    for (uint64_t e = near_ptr[a]; e < e1; ++e) {
        const uint32_t q = near_col[e];
        const uint32_t j1 = start[q + 1];
        // runs of 32 sources are summed on their own and then added in fp64: a long row of terms of
        // mixed sign loses fewer bits than with one running fp32 sum
        for (uint32_t j0 = start[q]; j0 < j1; j0 += 32) {
            const uint32_t je = min(j0 + 32u, j1);
            float run = 0.f;
#pragma unroll 4
            for (uint32_t j = j0; j < je; ++j) {
                float r2 = 0.f;
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    float diff = Xs[(int64_t)j * D + d] - xi[d];
                    r2 = fmaf(diff, diff, r2);
                }
                run = fmaf(__builtin_amdgcn_exp2f(r2 * nc2), bs[j], run);
            }
            acc += (double)run;
        }
    }
    if (active) ys[k] = accumulate ? ys[k] + (float)acc : (float)acc;
}

// ------------------------------------------------------------------------------------
// near field with the Gram matrix on the matrix cores.  In box units, relative to the centre
// of the target box (u = (x - centre)/l for a target, w = (y - centre)/l for a source) and with
// g = log2(e) l^2 / (2 gamma^2):
//   k(x,y) = exp2(-g|u|^2) * exp2( 2g u.w - g|w|^2 ).
// The second exponent for 32 sources x 32 targets is a dense contraction with inner
// dimension D+1: source vector (2g w_1..2g w_D, -g|w|^2), target vector (u_1..u_D, 1).  Each
// component is split into two fp16 numbers (hi = fp16(v), lo = fp16(v - hi): 22 significant
// bits) and the products hi*hi + hi*lo + lo*hi are laid side by side along the inner
// dimension, so one v_mfma_f32_32x32x16_f16 (fp32 accumulation, 8 passes) does the work of
// (D+2)/2 fp32 MFMAs of 16 passes each: 3(D+1) <= 16 terms for D <= 4, two instructions above.
// The dropped lo*lo term and the split are a perturbation of the coordinates by 2^-22 of a box
// edge.  exp2 and one FMA per pair stay on the vector ALU; exp2(-g|u|^2) is applied once per
// target.  A wavefront handles a run of <= 64 targets of one leaf box as two column blocks of
// 32; after the MFMA lane (n,h) holds the 16 sources 8(v/4)+4h+(v%4) of target column n, and
// the two halves are added with one shuffle at the end.
// Sources are cut from runs of rank-consecutive near boxes (contiguous points); rows beyond a
// run get zero coordinates and a norm term of -60000, so that their kernel value is
// exp2(-huge) = 0 whatever right-hand side is read for them.
// Used only while g is small (the caller checks it): the expanded square loses
// (|u|^2+|w|^2) g times the rounding unit in the exponent.
// ------------------------------------------------------------------------------------
typedef float f16v __attribute__((ext_vector_type(16)));
typedef _Float16 h8v __attribute__((ext_vector_type(8)));
struct __attribute__((packed, aligned(4))) float4u { float v[4]; };

// hi/lo fp16 split of NC components and the MFMA operand of one instruction:
//   term t of the inner dimension (t = 16 q + 8 h + e): kind = t / NC, component = t % NC
//   source side: (hi, hi, lo)[kind],  target side: (hi, lo, hi)[kind],  zero beyond 3 NC terms
template <int NC, bool SOURCE>
__device__ inline h8v split_operand(const float (&v)[NC], int q, int h) {
    _Float16 hi[NC], lo[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        hi[i] = (_Float16)v[i];
        lo[i] = (_Float16)(v[i] - (float)hi[i]);
    }
    h8v r;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        _Float16 val[2];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int t = 16 * q + 8 * hh + e;
            const int kind = t / NC, comp = t % NC;
            const bool use_lo = SOURCE ? kind == 2 : kind == 1;
            val[hh] = kind >= 3 ? (_Float16)0.f : (use_lo ? lo[comp] : hi[comp]);
        }
        r[e] = h ? val[1] : val[0];
    }
    return r;
}

typedef float f2v __attribute__((ext_vector_type(2)));
typedef _Float16 h2v __attribute__((ext_vector_type(2)));
typedef uint32_t u4v __attribute__((ext_vector_type(4)));

__device__ inline uint32_t pack_f16(float a, float b) {
    const h2v h = __builtin_convertvector((f2v){a, b}, h2v);
    return __builtin_bit_cast(uint32_t, h);
}
__device__ inline f2v unpack_f16(uint32_t v) { return __builtin_convertvector(__builtin_bit_cast(h2v, v), f2v); }

// source operand for four components (D = 3): the same layout as split_operand<4, true>,
// built from packed pairs.  Lane half 0 holds (hi, hi), lane half 1 (lo, 0).
__device__ inline h8v split_source4(const float (&w)[4], int h) {
    const uint32_t hi01 = pack_f16(w[0], w[1]), hi23 = pack_f16(w[2], w[3]);
    const f2v b01 = unpack_f16(hi01), b23 = unpack_f16(hi23);
    const uint32_t lo01 = pack_f16(w[0] - b01.x, w[1] - b01.y), lo23 = pack_f16(w[2] - b23.x, w[3] - b23.y);
    u4v r;
    r.x = h ? lo01 : hi01;
    r.y = h ? lo23 : hi23;
    r.z = h ? 0u : hi01;
    r.w = h ? 0u : hi23;
    return __builtin_bit_cast(h8v, r);
}

// target operand for four components (D = 3): the same layout as split_operand<4, false>, built
// from packed pairs.  Lane half 0 holds (hi, lo), lane half 1 (hi, 0).
__device__ inline h8v split_target4(const float (&u)[4], int h) {
    const uint32_t hi01 = pack_f16(u[0], u[1]), hi23 = pack_f16(u[2], u[3]);
    const f2v b01 = unpack_f16(hi01), b23 = unpack_f16(hi23);
    const uint32_t lo01 = pack_f16(u[0] - b01.x, u[1] - b01.y), lo23 = pack_f16(u[2] - b23.x, u[3] - b23.y);
    u4v r;
    r.x = hi01;
    r.y = hi23;
    r.z = h ? 0u : lo01;
    r.w = h ? 0u : lo23;
    return __builtin_bit_cast(h8v, r);
}

template <int D>
__global__ __launch_bounds__(256) void p2p_mfma_kernel(const float *__restrict__ Xt,
                                                       const uint32_t *__restrict__ startT,
                                                       const float *__restrict__ Xs, const float *__restrict__ bs,
                                                       const uint32_t *__restrict__ start,
                                                       const int32_t *__restrict__ cell,
                                                       const uint64_t *__restrict__ near_ptr,
                                                       const uint32_t *__restrict__ near_col,
                                                       const uint32_t *__restrict__ tile_box,
                                                       const uint32_t *__restrict__ tile_first, int64_t ntiles,
                                                       float g, float inv_l, CentreArg C, float *__restrict__ ys,
                                                       int accumulate) {
    constexpr int NC = D + 1;
    constexpr int NQ = (3 * NC + 15) / 16;   // MFMA instructions per 32 x 32 block
    const int lane = threadIdx.x & 63;
    const int64_t t = block_index() * 4 + (threadIdx.x >> 6);
    if (t >= ntiles) return;
    const uint32_t a = __builtin_amdgcn_readfirstlane(tile_box[t]);
    const uint32_t k0 = startT[a] + (uint32_t)(t - tile_first[a]) * 64u;
    const uint32_t kend = startT[a + 1];
    const bool two = __builtin_amdgcn_readfirstlane((int)(kend - k0)) > 32;
    const int nn = lane & 31, kk = lane >> 5;
    float ctr[D];
#pragma unroll
    for (int d = 0; d < D; ++d) ctr[d] = (float)(C.alpha[d] + ((double)cell[(int64_t)a * D + d] + 0.5) * C.edge);

    // B operands: the targets of the two column blocks
    h8v Bop[2][NQ];
    float ni[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const uint32_t kt = k0 + cb * 32 + nn;
        // unconditional loads (in bounds: Xs is padded by 64 points), masked by a factor so
        // that they are issued together and not one by one under a branch
        const float valid = kt < kend ? 1.f : 0.f;
        float u[NC];
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            u[d] = (Xt[(int64_t)kt * D + d] - ctr[d]) * inv_l * valid;
            s = fmaf(u[d], u[d], s);
        }
        u[D] = 1.f;
        ni[cb] = -g * s;
#pragma unroll
        for (int q = 0; q < NQ; ++q) Bop[cb][q] = split_operand<NC, false>(u, q, kk);
    }
    float acc0 = 0.f, acc1 = 0.f;
    const float g2l = 2.f * g * inv_l;
    const float nrm = -0.25f / g;

    // the blocks of 32 sources: near boxes with consecutive ranks are one contiguous run of
    // points, and blocks are cut from runs, not from single boxes, which wastes fewer rows.
    // (jb, je) is a block start and the end of its run; e walks the near list.
    uint64_t e = near_ptr[a];
    const uint64_t e1 = near_ptr[a + 1];
    auto next_run = [&](uint32_t &jb, uint32_t &je) {
        uint32_t q = near_col[e];
        jb = start[q];
        ++e;
        while (e < e1 && near_col[e] == q + 1) { ++q; ++e; }
        je = start[q + 1];
    };
    // the loads of a block: one source row per lane (both halves the same) and the right-hand
    // sides of the 16 sources this lane sees after the MFMA.  Always in bounds (64 points of
    // padding behind Xs and bs); rows at or beyond je are masked in block().
    auto load = [&](uint32_t jb, float (&x)[D], float4u (&bq)[4]) {
        const uint32_t j = jb + nn;
#pragma unroll
        for (int d = 0; d < D; ++d) x[d] = Xs[(int64_t)j * D + d];
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) bq[q4] = *reinterpret_cast<const float4u *>(bs + jb + 8 * q4 + 4 * kk);
    };
    auto block = [&](uint32_t jb, uint32_t je, const float (&x)[D], const float4u (&bq)[4]) {
        const bool live = jb + nn < je;
        float w[NC];
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            w[d] = (x[d] - ctr[d]) * (live ? g2l : 0.f);     // 2 g w_d
            s = fmaf(w[d], w[d], s);
        }
        w[D] = live ? s * nrm : -60000.f;              // -g |w|^2
        h8v Aop[NQ];
        if constexpr (NC == 4) {
            Aop[0] = split_source4(w, kk);
        } else {
#pragma unroll
            for (int qq = 0; qq < NQ; ++qq) Aop[qq] = split_operand<NC, true>(w, qq, kk);
        }
        f16v c0 = {0.f};
#pragma unroll
        for (int qq = 0; qq < NQ; ++qq) c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Aop[qq], Bop[0][qq], c0, 0, 0, 0);
        if (two) {
            f16v c1 = {0.f};
#pragma unroll
            for (int qq = 0; qq < NQ; ++qq) c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Aop[qq], Bop[1][qq], c1, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc0 = fmaf(__builtin_amdgcn_exp2f(c0[v]), bq[v >> 2].v[v & 3], acc0);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc1 = fmaf(__builtin_amdgcn_exp2f(c1[v]), bq[v >> 2].v[v & 3], acc1);
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc0 = fmaf(__builtin_amdgcn_exp2f(c0[v]), bq[v >> 2].v[v & 3], acc0);
        }
    };
    // A row can be empty (with the small field or the smooth field the box's own pair may be
    // handled elsewhere): nothing to add, and next_run must not read past the row.
    if (e == e1) {
        const uint32_t kt = k0 + kk * 32 + nn;
        if (kt < kend) ys[kt] = accumulate ? ys[kt] : 0.f;
        return;
    }
    // two register sets in turn: the loads of the next block are in flight while the current
    // one is worked on.
    float xa[D], xb[D];
    float4u ba[4], bb[4];
    uint32_t jba, jea, jbb, jeb;
    next_run(jba, jea);
    load(jba, xa, ba);
    for (;;) {
        jbb = jba + 32;
        jeb = jea;
        bool more = true;
        if (jbb >= jea) {
            if (e < e1) next_run(jbb, jeb);
            else more = false;
        }
        load(more ? jbb : jba, xb, bb);     // unconditional: a fixed number of loads in flight
        block(jba, jea, xa, ba);
        if (!more) break;
        jba = jbb + 32;
        jea = jeb;
        if (jba >= jeb) {
            if (e < e1) next_run(jba, jea);
            else more = false;
        }
        load(more ? jba : jbb, xa, ba);
        block(jbb, jeb, xb, bb);
        if (!more) break;
    }
    acc0 += __shfl_xor(acc0, 32, 64);
    acc1 += __shfl_xor(acc1, 32, 64);
    const float res = kk ? __builtin_amdgcn_exp2f(ni[1]) * acc1 : __builtin_amdgcn_exp2f(ni[0]) * acc0;
    const uint32_t kt = k0 + kk * 32 + nn;
    if (kt < kend) ys[kt] = accumulate ? ys[kt] + res : res;
}

// The near-field kernel for D = 3.  The sources of a target tile are the points of its near
// boxes, taken as ONE dense sequence: lane r of the wavefront holds (first point, length,
// running offsets) of near box r, and the source at sequence position p is found from that
// table with wave-uniform lane reads, so steps of 64 sources are full except the last one.
// Source operands are prepared for 64 sources at a time: lane l loads the source at position
// w0 + l, splits its four components (2g w_x, 2g w_y, 2g w_z, -g|w|^2) into packed fp16 pairs
// hi01, hi23, lo01, lo23, and one v_permlane32_swap per pair turns (hi, lo) into the operand
// registers of two blocks of 32 sources at once:
//   swap(hi, lo): hi' = [hi of sources 0-31 | lo of sources 0-31]   -> block A, both lane halves
//                 lo' = [hi of sources 32-63 | lo of sources 32-63] -> block B
// Inner dimension of the MFMA (k = 8 half + e): source side half 0 = (hi, hi), half 1 = (lo, lo);
// target side half 0 = (hi, lo), half 1 = (hi, 0): hi*hi + hi*lo + lo*hi, the fourth product
// meets a zero.  The right-hand sides of a step pass through 64 floats of LDS per wavefront
// (written by the lane that owns the source, read as the 16 values a lane needs per block).
// SPLIT: a problem with few target tiles and long rows (few targets against many sources) gives
// every tile to `nsplit` wavefronts; wavefront s of a tile takes the s-th slice (a multiple of 64
// positions) of the source sequence of every round and writes its sums to part[s][target]; they
// are added in ascending s by p2p_split_sum_kernel.
// MB > 1: MB right-hand sides at once (MA.bs[j] -> MA.ys[j]); the exponents and the exponentials of a
// block are formed once and every right-hand side adds its own 16 multiply-adds per lane, so the
// dominant cost of the near field is shared by the columns.
struct MultiArg {
    const float *bs[4];
    float *ys[4];
};

template <bool SPLIT, int MB>
__global__ __launch_bounds__(256) void p2p_gram3_kernel(const float *__restrict__ Xt,
                                                        const uint32_t *__restrict__ startT,
                                                        const float *__restrict__ Xs, const float *__restrict__ bs,
                                                        const uint32_t *__restrict__ start,
                                                        const int32_t *__restrict__ cell,
                                                        const uint64_t *__restrict__ near_ptr,
                                                        const uint32_t *__restrict__ near_col,
                                                        const uint32_t *__restrict__ tile_box,
                                                        const uint32_t *__restrict__ tile_first, int64_t ntiles,
                                                        float g, float inv_l, CentreArg C, float *__restrict__ ys,
                                                        int accumulate, int nsplit, int64_t ntargets,
                                                        float *__restrict__ part, MultiArg MA,
                                                        const uint8_t *__restrict__ paired) {
    constexpr int D = 3, NC = 4;
    static_assert(MB >= 1 && MB <= 4 && !(SPLIT && MB > 1), "unsupported variant");
    __shared__ __attribute__((aligned(16))) float bbuf[4][MB * 64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int64_t t = block_index() * 4 + wv;
    int slice = 0;
    if constexpr (SPLIT) {
        if (t >= ntiles * nsplit) return;
        const int64_t tile = t / nsplit;
        slice = (int)(t - tile * nsplit);
        t = tile;
    } else {
        if (t >= ntiles) return;
    }
    const uint32_t a = __builtin_amdgcn_readfirstlane(tile_box[t]);
    // paired (or null): boxes whose first run of targets is worked by p2p_gram3_pair_kernel; the tile list
    // then starts at their second run
    const uint32_t k0 = startT[a] + ((uint32_t)(t - tile_first[a]) + (paired && paired[a] ? 1u : 0u)) * 64u;
    const uint32_t kend = startT[a + 1];
    const int ntg = __builtin_amdgcn_readfirstlane((int)(kend - k0));   // targets of the tile (wave-uniform)
    const int nn = lane & 31, kk = lane >> 5;
    float ctr[D];
#pragma unroll
    for (int d = 0; d < D; ++d) ctr[d] = (float)(C.alpha[d] + ((double)cell[(int64_t)a * D + d] + 0.5) * C.edge);

    // B operands: the targets of the two column blocks
    h8v Bop[2];
    float ni[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const uint32_t kt = k0 + cb * 32 + nn;
        const float valid = kt < kend ? 1.f : 0.f;   // loads are in bounds (padding), masked by a factor
        float u[NC];
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            u[d] = (Xt[(int64_t)kt * D + d] - ctr[d]) * inv_l * valid;
            s = fmaf(u[d], u[d], s);
        }
        u[D] = 1.f;
        ni[cb] = -g * s;
        Bop[cb] = split_target4(u, kk);
    }
    float acc0 = 0.f, acc1 = 0.f;
    float accm0[MB], accm1[MB];   // MB > 1: one pair of accumulators per right-hand side
#pragma unroll
    for (int j = 0; j < MB; ++j) accm0[j] = accm1[j] = 0.f;
    const float g2l = 2.f * g * inv_l;
    const float nrm = -0.25f / g;
    float *bw = bbuf[wv];

    // operands of the two blocks of 32 sources of a step.  A lane whose position lies behind the
    // sequence holds the last source again (a near point like the others: finite exponent) and
    // its right-hand side is zero.
    auto prepare = [&](const float (&x)[D], h8v &opA, h8v &opB) {
        float w[NC];
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            w[d] = (x[d] - ctr[d]) * g2l;                    // 2 g w_d
            s = fmaf(w[d], w[d], s);
        }
        w[D] = s * nrm;                                      // -g |w|^2
        const uint32_t hi01 = pack_f16(w[0], w[1]), hi23 = pack_f16(w[2], w[3]);
        const f2v b01 = unpack_f16(hi01), b23 = unpack_f16(hi23);
        const uint32_t lo01 = pack_f16(w[0] - b01.x, w[1] - b01.y), lo23 = pack_f16(w[2] - b23.x, w[3] - b23.y);
        const auto s01 = __builtin_amdgcn_permlane32_swap(hi01, lo01, false, false);
        const auto s23 = __builtin_amdgcn_permlane32_swap(hi23, lo23, false, false);
        u4v ra, rb;
        ra.x = s01[0]; ra.y = s23[0]; ra.z = s01[0]; ra.w = s23[0];
        rb.x = s01[1]; rb.y = s23[1]; rb.z = s01[1]; rb.w = s23[1];
        opA = __builtin_bit_cast(h8v, ra);
        opB = __builtin_bit_cast(h8v, rb);
    };
    // one block of 32 sources against the tile; bq = right-hand sides at bw[first .. first + 31].
    // (The two column blocks are summed in differently shaped code on purpose: identical
    // sequences get merged by the compiler into one that addresses the accumulators through
    // scratch memory.)
    auto block = [&](const h8v &op, int first) {
        if constexpr (MB > 1) {
            // the exponentials once, then 16 multiply-adds per right-hand side and column block
            f16v e0 = {0.f}, e1 = {0.f};
            e0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(op, Bop[0], e0, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 16; ++v) e0[v] = __builtin_amdgcn_exp2f(e0[v]);
            if (ntg > 32) {
                e1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(op, Bop[1], e1, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; ++v) e1[v] = __builtin_amdgcn_exp2f(e1[v]);
            }
#pragma unroll
            for (int j = 0; j < MB; ++j) {
                float4 bq[4];
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    bq[q4] = *reinterpret_cast<const float4 *>(bw + j * 64 + first + 8 * q4 + 4 * kk);
                const float *bf = reinterpret_cast<const float *>(bq);
#pragma unroll
                for (int v = 0; v < 16; ++v) accm0[j] = fmaf(e0[v], bf[v], accm0[j]);
                if (ntg > 32) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) accm1[j] = fmaf(e1[v], bf[v], accm1[j]);
                }
            }
            return;
        }
        float4 bq[4];
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) bq[q4] = *reinterpret_cast<const float4 *>(bw + first + 8 * q4 + 4 * kk);
        const float *bf = reinterpret_cast<const float *>(bq);
        f16v c0 = {0.f};
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(op, Bop[0], c0, 0, 0, 0);
        // the test is made on a scalar register at each use: kept as a lane mask across the loop it
        // costs two vector instructions per step
        int nt2 = ntg;
        asm volatile("" : "+s"(nt2));
        if (nt2 > 32) {
            f16v c1 = {0.f};
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(op, Bop[1], c1, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc0 = fmaf(__builtin_amdgcn_exp2f(c0[v]), bf[v], acc0);
#pragma unroll
            for (int v = 15; v >= 0; --v) acc1 = fmaf(__builtin_amdgcn_exp2f(c1[v]), bf[v], acc1);
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc0 = fmaf(__builtin_amdgcn_exp2f(c0[v]), bf[v], acc0);
        }
    };

    const uint64_t e0 = near_ptr[a], e1 = near_ptr[a + 1];
    for (uint64_t er = e0; er < e1; er += 64) {   // rounds of up to 64 near boxes (one round with far ratio 2)
        const int m = (int)(e1 - er < 64 ? e1 - er : 64);
        uint32_t sfirst = 0, slen = 0;
        if (lane < m) {
            const uint32_t q = near_col[er + lane];
            sfirst = start[q];
            slen = start[q + 1] - sfirst;
        }
        const uint32_t cend = wave_incl_scan_u32(slen);   // inclusive running sum of the lengths over the lanes
        const uint32_t cbeg = cend - slen;
        const uint32_t delta = sfirst - cbeg;   // position -> source index inside this lane's box (mod 2^32)
        uint32_t S = __builtin_amdgcn_readlane(cend, 63);   // sources of this round
        uint32_t wbeg = 0;                                   // this wavefront's positions: [wbeg, S)
        if constexpr (SPLIT) {
            const uint32_t per = ((S + (uint32_t)nsplit - 1) / (uint32_t)nsplit + 63u) & ~63u;
            const uint64_t lo = (uint64_t)slice * per;
            wbeg = lo < S ? (uint32_t)lo : S;
            S = (uint64_t)wbeg + per < S ? wbeg + per : S;
            // wave-uniform, but derived from the wavefront's number: kept in scalar registers by force
            wbeg = __builtin_amdgcn_readfirstlane(wbeg);
            S = __builtin_amdgcn_readfirstlane(S);
        }
        if (wbeg >= S) continue;
        int r = 0;   // first near box that reaches into the current window (wave-uniform)
        // Source index of position w0 + lane; positions from S on take the last source of the
        // sequence, so every index is in bounds.  Box r holds w0 (cbeg <= w0 < cend), so it is the
        // box of every position until a later box begins at or before the position; a box without
        // points is overridden by its successor, which begins at the same position.
        auto locate = [&](uint32_t w0) {
            const uint32_t p = min(w0 + (uint32_t)lane, S - 1u);
            while ((uint32_t)__builtin_amdgcn_readlane(cend, r) <= w0) ++r;   // ends: w0 < S <= cend of lane 63
            uint32_t src = p + (uint32_t)__builtin_amdgcn_readlane(delta, r);
            for (int rr = r + 1; rr < m; ++rr) {
                const uint32_t c0 = __builtin_amdgcn_readlane(cbeg, rr);
                if (c0 >= w0 + 64) break;
                const uint32_t dl = __builtin_amdgcn_readlane(delta, rr);
                src = p >= c0 ? p + dl : src;
            }
            return src;
        };
        // Two register sets take turns as "current" and "next" step (no copies at the end of a step): the loads
        // of the next step are in flight during the current one; the last step loads its own sources again,
        // so the number of loads in flight is fixed.
        auto fetch = [&](uint32_t w0, float (&x)[D], float &b1, float (&bm)[MB]) __attribute__((always_inline)) {
            const uint32_t src = locate(w0);
#pragma unroll
            for (int d = 0; d < D; ++d) x[d] = Xs[(int64_t)src * D + d];
            if constexpr (MB > 1) {
#pragma unroll
                for (int j = 0; j < MB; ++j) bm[j] = MA.bs[j][src];
            } else {
                b1 = bs[src];
            }
        };
        auto step = [&](uint32_t w0, const float (&xc)[D], float bc, float (&bcm)[MB], float (&xnext)[D], float &bnext,
                        float (&bnextm)[MB]) __attribute__((always_inline)) {
            fetch(w0 + 64 < S ? w0 + 64 : w0, xnext, bnext, bnextm);
            if (w0 + 64 > S) {   // last step only: the positions behind the sequence get weight zero
                asm volatile("");   // keeps this a branch: as selects it costs every step three instructions
                const bool live = w0 + lane < S;
                bc = live ? bc : 0.f;
#pragma unroll
                for (int j = 0; j < MB; ++j) bcm[j] = live ? bcm[j] : 0.f;
            }
            __builtin_amdgcn_wave_barrier();
            if constexpr (MB > 1) {
#pragma unroll
                for (int j = 0; j < MB; ++j) bw[j * 64 + lane] = bcm[j];
            } else {
                bw[lane] = bc;
            }
            __builtin_amdgcn_wave_barrier();   // LDS operations of a wavefront complete in order
            h8v opA, opB;
            prepare(xc, opA, opB);
            block(opA, 0);
            if (w0 + 32 < S) block(opB, 32);
        };
        float xa[D], xb[D], ba = 0.f, bb = 0.f;
        float bam[MB], bbm[MB];
#pragma unroll
        for (int j = 0; j < MB; ++j) bam[j] = bbm[j] = 0.f;
        fetch(wbeg, xa, ba, bam);
        for (uint32_t w0 = wbeg;;) {
            step(w0, xa, ba, bam, xb, bb, bbm);
            w0 += 64;
            if (w0 >= S) break;
            step(w0, xb, bb, bbm, xa, ba, bam);
            w0 += 64;
            if (w0 >= S) break;
        }
    }
    if constexpr (MB > 1) {
        const uint32_t kt = k0 + kk * 32 + nn;
        const float scale = __builtin_amdgcn_exp2f(kk ? ni[1] : ni[0]);
#pragma unroll
        for (int j = 0; j < MB; ++j) {
            const float a0 = accm0[j] + __shfl_xor(accm0[j], 32, 64), a1 = accm1[j] + __shfl_xor(accm1[j], 32, 64);
            if (kt < kend) MA.ys[j][kt] = scale * (kk ? a1 : a0);
        }
        return;
    }
    acc0 += __shfl_xor(acc0, 32, 64);
    acc1 += __shfl_xor(acc1, 32, 64);
    const float res = kk ? __builtin_amdgcn_exp2f(ni[1]) * acc1 : __builtin_amdgcn_exp2f(ni[0]) * acc0;
    const uint32_t kt = k0 + kk * 32 + nn;
    if constexpr (SPLIT) {
        if (kt < kend) part[(int64_t)slice * ntargets + kt] = res;
    } else {
        if (kt < kend) ys[kt] = accumulate ? ys[kt] + res : res;
    }
}

// The 3-D Gram near field for PAIRS of target tiles.  Two leaf boxes a and a + 1 with the same parent and
// cells next to each other share most of their near boxes (18 of 27 with far ratio 2), and the cost of a step
// of p2p_gram3_kernel that is not exponentials and multiply-adds (finding and loading 64 sources, preparing
// their operands) does not depend on the number of target columns.  One wavefront takes the first run of
// targets of both boxes: coordinates are relative to the midpoint of the two box centres, and the source
// sequence is cut in three segments,
//   [ boxes near both | boxes near a only | boxes near a + 1 only ],
// each walked like the sequence of p2p_gram3_kernel; the first segment is worked against four column blocks.
// The segments come from the two near rows (at most 32 entries each: lanes 0-31 hold the row of a, lanes 32-63
// that of a + 1): an entry of a's row is also near a + 1 iff its squared cell offset from a + 1 is below the
// far threshold T (the integer rule that built the rows), and the copies in the row of a + 1 are dropped.
// Within a segment boxes keep their list order.
__global__ __launch_bounds__(256) void p2p_gram3_pair_kernel(const float *__restrict__ Xs,
                                                             const uint32_t *__restrict__ start,
                                                             const float *__restrict__ bs,
                                                             const int32_t *__restrict__ cell,
                                                             const uint64_t *__restrict__ near_ptr,
                                                             const uint32_t *__restrict__ near_col,
                                                             const uint32_t *__restrict__ pair_box, int64_t npairs,
                                                             int T, float g, float inv_l, CentreArg C,
                                                             float *__restrict__ ys) {
    constexpr int D = 3, NC = 4;
    __shared__ __attribute__((aligned(16))) float bbuf[4][64];
    __shared__ uint32_t tab_first[4][64], tab_len[4][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int64_t t = block_index() * 4 + wv;
    if (t >= npairs) return;
    const uint32_t a = __builtin_amdgcn_readfirstlane(pair_box[t]);   // the pair is (a, a + 1)
    const int nn = lane & 31, kk = lane >> 5;
    int32_t ca[D], eo[D];   // cell of a, and the cell of a + 1 relative to it
    float ctr[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        ca[d] = cell[(int64_t)a * D + d];
        eo[d] = cell[(int64_t)(a + 1) * D + d] - ca[d];
        ctr[d] = (float)(C.alpha[d] + ((double)ca[d] + 0.5 + 0.5 * (double)eo[d]) * C.edge);
    }
    const uint32_t kA = start[a], kB = start[a + 1], kBe = start[a + 2];
    const int ntA = __builtin_amdgcn_readfirstlane((int)min(kB - kA, 64u));    // targets of the two tiles
    const int ntB = __builtin_amdgcn_readfirstlane((int)min(kBe - kB, 64u));

    // B operands: column blocks 0, 1 are the targets of a, blocks 2, 3 those of a + 1
    h8v Bop[4];
    float ni[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const int idx = (cb & 1) * 32 + nn;
        const uint32_t kt = (cb < 2 ? kA : kB) + (uint32_t)idx;
        const float valid = idx < (cb < 2 ? ntA : ntB) ? 1.f : 0.f;   // loads are in bounds (padding), masked by a factor
        float u[NC];
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            u[d] = (Xs[(int64_t)kt * D + d] - ctr[d]) * inv_l * valid;
            s = fmaf(u[d], u[d], s);
        }
        u[D] = 1.f;
        ni[cb] = -g * s;
        Bop[cb] = split_target4(u, kk);
    }

    // the table of the source boxes: lane = position in [both | a only | a + 1 only]
    int nboth, nonly_a, m;
    uint32_t sfirst, slen;
    {
        const bool of_a = lane < 32;
        const uint64_t e0 = near_ptr[a], e1 = near_ptr[a + 1], e2 = near_ptr[a + 2];
        const int len = (int)(of_a ? e1 - e0 : e2 - e1);
        const bool have = (lane & 31) < len;
        const uint32_t q = have ? near_col[(of_a ? e0 : e1) + (uint64_t)(lane & 31)] : a;
        int d2 = 0;   // squared cell offset of q from the OTHER box of the pair
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int o = cell[(int64_t)q * D + d] - ca[d] - (of_a ? eo[d] : 0);
            d2 += o * o;
        }
        const bool other = d2 < T;
        const bool is_both = have && of_a && other, is_a = have && of_a && !other, is_b = have && !of_a && !other;
        const uint64_t mboth = __ballot(is_both), ma = __ballot(is_a), mb = __ballot(is_b);
        const uint64_t below = (1ull << lane) - 1ull;
        nboth = __popcll(mboth);
        nonly_a = __popcll(ma);
        m = nboth + nonly_a + __popcll(mb);
        const int slot = is_both ? __popcll(mboth & below)
                       : is_a    ? nboth + __popcll(ma & below)
                                 : nboth + nonly_a + __popcll(mb & below);
        const uint32_t f = start[q], l = start[q + 1] - f;
        tab_first[wv][lane] = 0u;
        tab_len[wv][lane] = 0u;
        __builtin_amdgcn_wave_barrier();   // LDS operations of a wavefront complete in order
        if (is_both || is_a || is_b) {
            tab_first[wv][slot] = f;
            tab_len[wv][slot] = l;
        }
        __builtin_amdgcn_wave_barrier();
        sfirst = tab_first[wv][lane];
        slen = tab_len[wv][lane];
    }
    const uint32_t cend = wave_incl_scan_u32(slen);   // inclusive running sum of the lengths over the lanes
    const uint32_t cbeg = cend - slen;
    const uint32_t delta = sfirst - cbeg;   // position -> source index inside this lane's box (mod 2^32)
    const uint32_t S1 = nboth > 0 ? (uint32_t)__builtin_amdgcn_readlane(cend, nboth - 1) : 0u;
    const uint32_t S2 = nboth + nonly_a > 0 ? (uint32_t)__builtin_amdgcn_readlane(cend, nboth + nonly_a - 1) : 0u;
    const uint32_t S3 = __builtin_amdgcn_readlane(cend, 63);

    float accA0 = 0.f, accA1 = 0.f, accB0 = 0.f, accB1 = 0.f;
    const float g2l = 2.f * g * inv_l;
    const float nrm = -0.25f / g;
    float *bw = bbuf[wv];
    int r = 0;   // first box of the table that reaches into the current window (wave-uniform, only grows)

    // operands of the two blocks of 32 sources of a step, as in p2p_gram3_kernel
    auto prepare = [&](const float (&x)[D], h8v &opA, h8v &opB) __attribute__((always_inline)) {
        float w[NC];
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            w[d] = (x[d] - ctr[d]) * g2l;                    // 2 g w_d
            s = fmaf(w[d], w[d], s);
        }
        w[D] = s * nrm;                                      // -g |w|^2
        const uint32_t hi01 = pack_f16(w[0], w[1]), hi23 = pack_f16(w[2], w[3]);
        const f2v b01 = unpack_f16(hi01), b23 = unpack_f16(hi23);
        const uint32_t lo01 = pack_f16(w[0] - b01.x, w[1] - b01.y), lo23 = pack_f16(w[2] - b23.x, w[3] - b23.y);
        const auto s01 = __builtin_amdgcn_permlane32_swap(hi01, lo01, false, false);
        const auto s23 = __builtin_amdgcn_permlane32_swap(hi23, lo23, false, false);
        u4v ra, rb;
        ra.x = s01[0]; ra.y = s23[0]; ra.z = s01[0]; ra.w = s23[0];
        rb.x = s01[1]; rb.y = s23[1]; rb.z = s01[1]; rb.w = s23[1];
        opA = __builtin_bit_cast(h8v, ra);
        opB = __builtin_bit_cast(h8v, rb);
    };
    // one block of 32 sources against the column blocks of one tile
    auto columns = [&](const h8v &op, const float *bf, const h8v &B0, const h8v &B1, int nt, float &acc0,
                       float &acc1) __attribute__((always_inline)) {
        f16v c0 = {0.f};
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(op, B0, c0, 0, 0, 0);
        int nt2 = nt;
        asm volatile("" : "+s"(nt2));   // the test on a scalar register at each use, not on a kept lane mask
        if (nt2 > 32) {
            f16v c1 = {0.f};
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(op, B1, c1, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc0 = fmaf(__builtin_amdgcn_exp2f(c0[v]), bf[v], acc0);
#pragma unroll
            for (int v = 15; v >= 0; --v) acc1 = fmaf(__builtin_amdgcn_exp2f(c1[v]), bf[v], acc1);
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc0 = fmaf(__builtin_amdgcn_exp2f(c0[v]), bf[v], acc0);
        }
    };
    // the positions [wbeg, S) of the sequence against the tiles in `which` (1: a, 2: a + 1, 3: both)
    auto segment = [&](uint32_t wbeg, uint32_t S, auto which) __attribute__((always_inline)) {
        constexpr int W = decltype(which)::value;
        if (wbeg >= S) return;
        // source index of position w0 + lane, as in p2p_gram3_kernel; positions from S on take the last source
        // of the segment (w0 < S <= cend of lane 63 ends the search)
        auto locate = [&](uint32_t w0) __attribute__((always_inline)) {
            const uint32_t p = min(w0 + (uint32_t)lane, S - 1u);
            while ((uint32_t)__builtin_amdgcn_readlane(cend, r) <= w0) ++r;
            uint32_t src = p + (uint32_t)__builtin_amdgcn_readlane(delta, r);
            for (int rr = r + 1; rr < m; ++rr) {
                const uint32_t c0 = __builtin_amdgcn_readlane(cbeg, rr);
                if (c0 >= w0 + 64) break;
                const uint32_t dl = __builtin_amdgcn_readlane(delta, rr);
                src = p >= c0 ? p + dl : src;
            }
            return src;
        };
        // two register sets take turns as current and next step, as in p2p_gram3_kernel
        auto fetch = [&](uint32_t w0, float (&x)[D], float &b1) __attribute__((always_inline)) {
            const uint32_t src = locate(w0);
#pragma unroll
            for (int d = 0; d < D; ++d) x[d] = Xs[(int64_t)src * D + d];
            b1 = bs[src];
        };
        auto step = [&](uint32_t w0, const float (&xc)[D], float bc, float (&xnext)[D], float &bnext)
                        __attribute__((always_inline)) {
            fetch(w0 + 64 < S ? w0 + 64 : w0, xnext, bnext);
            if (w0 + 64 > S) {   // last step only: the positions behind the segment get weight zero
                asm volatile("");
                bc = w0 + lane < S ? bc : 0.f;
            }
            __builtin_amdgcn_wave_barrier();
            bw[lane] = bc;
            __builtin_amdgcn_wave_barrier();   // LDS operations of a wavefront complete in order
            h8v opA, opB;
            prepare(xc, opA, opB);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                if (half == 1 && w0 + 32 >= S) break;
                float4 bq[4];
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    bq[q4] = *reinterpret_cast<const float4 *>(bw + 32 * half + 8 * q4 + 4 * kk);
                const float *bf = reinterpret_cast<const float *>(bq);
                const h8v &op = half ? opB : opA;
                if constexpr ((W & 1) != 0) columns(op, bf, Bop[0], Bop[1], ntA, accA0, accA1);
                if constexpr ((W & 2) != 0) columns(op, bf, Bop[2], Bop[3], ntB, accB0, accB1);
            }
        };
        float xa[D], xb[D], ba, bb;
        fetch(wbeg, xa, ba);
        for (uint32_t w0 = wbeg;;) {
            step(w0, xa, ba, xb, bb);
            w0 += 64;
            if (w0 >= S) break;
            step(w0, xb, bb, xa, ba);
            w0 += 64;
            if (w0 >= S) break;
        }
    };
    segment(0u, S1, std::integral_constant<int, 3>{});
    segment(S1, S2, std::integral_constant<int, 1>{});
    segment(S2, S3, std::integral_constant<int, 2>{});

    accA0 += __shfl_xor(accA0, 32, 64);
    accA1 += __shfl_xor(accA1, 32, 64);
    accB0 += __shfl_xor(accB0, 32, 64);
    accB1 += __shfl_xor(accB1, 32, 64);
    const int idx = kk * 32 + nn;
    const float resA = kk ? __builtin_amdgcn_exp2f(ni[1]) * accA1 : __builtin_amdgcn_exp2f(ni[0]) * accA0;
    const float resB = kk ? __builtin_amdgcn_exp2f(ni[3]) * accB1 : __builtin_amdgcn_exp2f(ni[2]) * accB0;
    if (idx < ntA) ys[kA + (uint32_t)idx] = resA;
    if (idx < ntB) ys[kB + (uint32_t)idx] = resB;
}

// sums of the slices of a split near-field launch, in ascending slice order
__global__ __launch_bounds__(256) void p2p_split_sum_kernel(const float *__restrict__ part, int nsplit, int64_t n,
                                                            float *__restrict__ ys, int accumulate) {
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= n) return;
    float s = accumulate ? ys[k] : 0.f;
    for (int j = 0; j < nsplit; ++j) s += part[(int64_t)j * n + k];
    ys[k] = s;
}

// Direct sums for the small-field pairs of a depth (Sec. 4.2): both boxes of a pair hold few
// points, so neither a lane per target nor blocks of 32 x 32 would be filled.  Here lane =
// source: the sources of a target box's row are taken as one dense sequence over its boxes
// (the lane-held segment table of p2p_gram3_kernel), 64 per step, and a wavefront handles a run
// of at most SMALL_TT targets of one box, whose coordinates are wave-uniform.  Every lane keeps
// one partial sum per target; they are added across the lanes once, at the end.  Differences
// are formed directly (the pairs may be several boxes apart).  The result is added to ys
// (accumulate) or written.  The same kernel takes the overflow tiles of the near field of the last
// depth (overflow != 0): one tile per listed box, the targets behind its last full run of 64.
template <int D>
constexpr int small_tt() { return D <= 4 ? 16 : 8; }

template <int D, int TT>
__global__ __launch_bounds__(256) void p2p_small_kernel(const float *__restrict__ Xt,
                                                        const uint32_t *__restrict__ startT,
                                                        const float *__restrict__ Xs, const float *__restrict__ bs,
                                                        const uint32_t *__restrict__ start,
                                                        const uint64_t *__restrict__ row_ptr,
                                                        const uint32_t *__restrict__ cols,
                                                        const uint32_t *__restrict__ tile_box,
                                                        const uint32_t *__restrict__ tile_first, int64_t ntiles,
                                                        float nc2, float *__restrict__ ys, int overflow, int accumulate) {
    const int lane = threadIdx.x & 63;
    const int64_t t = block_index() * 4 + (threadIdx.x >> 6);
    if (t >= ntiles) return;
    const uint32_t a = __builtin_amdgcn_readfirstlane(tile_box[t]);
    const uint32_t kend = startT[a + 1];
    const uint32_t k0 = overflow ? startT[a] + ((kend - startT[a]) & ~63u)
                                 : startT[a] + (uint32_t)(t - tile_first[a]) * (uint32_t)TT;
    const int nt = (int)(kend - k0 < (uint32_t)TT ? kend - k0 : (uint32_t)TT);   // wave-uniform
    float xt[TT][D];   // target coordinates, wave-uniform (rows beyond nt repeat an in-bounds point)
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const uint32_t kt = k0 + (uint32_t)(tt < nt ? tt : 0);
#pragma unroll
        for (int d = 0; d < D; ++d) xt[tt][d] = Xt[(int64_t)kt * D + d];
    }
    float acc[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) acc[tt] = 0.f;

    const uint64_t e0 = row_ptr[a], e1 = row_ptr[a + 1];
    for (uint64_t er = e0; er < e1; er += 64) {   // rounds of up to 64 boxes of the row
        const int m = (int)(e1 - er < 64 ? e1 - er : 64);
        uint32_t sfirst = 0, slen = 0;
        if (lane < m) {
            const uint32_t q = cols[er + lane];
            sfirst = start[q];
            slen = start[q + 1] - sfirst;
        }
        const uint32_t cend = wave_incl_scan_u32(slen);   // inclusive running sum of the lengths over the lanes
        const uint32_t cbeg = cend - slen;
        const uint32_t delta = sfirst - cbeg;   // position -> source index inside this lane's box (mod 2^32)
        const uint32_t S = __builtin_amdgcn_readlane(cend, 63);
        if (S == 0) continue;
        int r = 0;
        // source index of position w0 + lane, as in p2p_gram3_kernel (positions from S on take the
        // last source of the sequence)
        auto locate = [&](uint32_t w0) {
            const uint32_t p = min(w0 + (uint32_t)lane, S - 1u);
            while ((uint32_t)__builtin_amdgcn_readlane(cend, r) <= w0) ++r;   // ends: w0 < S = cend of lane 63
            uint32_t src = p + (uint32_t)__builtin_amdgcn_readlane(delta, r);
            for (int rr = r + 1; rr < m; ++rr) {
                const uint32_t c0 = __builtin_amdgcn_readlane(cbeg, rr);
                if (c0 >= w0 + 64) break;
                const uint32_t dl = __builtin_amdgcn_readlane(delta, rr);
                src = p >= c0 ? p + dl : src;
            }
            return src;
        };
        float xn[D], bn;
        {
            const uint32_t src = locate(0);
#pragma unroll
            for (int d = 0; d < D; ++d) xn[d] = Xs[(int64_t)src * D + d];
            bn = bs[src];
        }
        for (uint32_t w0 = 0; w0 < S; w0 += 64) {
            float x[D];
#pragma unroll
            for (int d = 0; d < D; ++d) x[d] = xn[d];
            float bv = bn;
            if (w0 + 64 > S) {      // last step only: positions behind the sequence contribute nothing
                asm volatile("");   // keeps this a branch (as a select it costs every step three instructions)
                bv = w0 + lane < S ? bv : 0.f;
            }
            // the loads of the next step are in flight during this one (the last step loads its own
            // sources again, so the number of loads in flight is fixed)
            const uint32_t nsrc = locate(w0 + 64 < S ? w0 + 64 : w0);
#pragma unroll
            for (int d = 0; d < D; ++d) xn[d] = Xs[(int64_t)nsrc * D + d];
            bn = bs[nsrc];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                if (tt < nt) {
                    float r2 = 0.f;
#pragma unroll
                    for (int d = 0; d < D; ++d) {
                        const float df = x[d] - xt[tt][d];
                        r2 = fmaf(df, df, r2);
                    }
                    acc[tt] = fmaf(__builtin_amdgcn_exp2f(r2 * nc2), bv, acc[tt]);
                }
            }
        }
    }
    // sums over the lanes; lane tt keeps the total of target tt
    float res = 0.f;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        if (tt < nt) {
            float v = acc[tt];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
            if (lane == tt) res = v;
        }
    }
    if (lane < nt) ys[k0 + lane] = accumulate ? ys[k0 + lane] + res : res;
}

// exact product, all pairs (Sec. 2, KeOps paragraph): lane = target (rows of X, nx of them), the
// sources (rows of Y, ny of them, weights b) wave-uniform; X == Y for one point set
template <int D>
__global__ __launch_bounds__(64) void direct_kernel(const float *__restrict__ X, int64_t nx,
                                                    const float *__restrict__ Y, const float *__restrict__ b,
                                                    int64_t n, float nc2, float *__restrict__ y) {
    const int64_t i = (int64_t)blockIdx.x * 64 + threadIdx.x;
    const bool active = i < nx;
    float xi[D];
#pragma unroll
    for (int d = 0; d < D; ++d) xi[d] = active ? X[i * D + d] : 0.f;
    double acc = 0.0;
    for (int64_t j0 = 0; j0 < n; j0 += 32) {   // runs of 32 sources summed on their own, then added in fp64
        const int64_t je = min(j0 + 32, n);
        float run = 0.f;
#pragma unroll 4
        for (int64_t j = j0; j < je; ++j) {
            float r2 = 0.f;
#pragma unroll
            for (int d = 0; d < D; ++d) {
                float diff = Y[j * D + d] - xi[d];
                r2 = fmaf(diff, diff, r2);
            }
            run = fmaf(__builtin_amdgcn_exp2f(r2 * nc2), b[j], run);
        }
        acc += (double)run;
    }
    if (active) y[i] = (float)acc;
}

// exact rows in fp64: lane = row, blockIdx.y = slice of the sources; partial sums per slice
template <int D>
__global__ __launch_bounds__(64) void rows_f64_kernel(const float *__restrict__ X, const float *__restrict__ Y,
                                                      const float *__restrict__ b, int64_t n,
                                                      const int64_t *__restrict__ rows, int64_t m,
                                                      double nc, double *__restrict__ part) {
    const int64_t a = (int64_t)blockIdx.x * 64 + threadIdx.x;
    const bool active = a < m;
    double xi[D];
    const int64_t i = active ? rows[a] : 0;
#pragma unroll
    for (int d = 0; d < D; ++d) xi[d] = (double)X[i * D + d];
    const int64_t per = (n + gridDim.y - 1) / gridDim.y;
    const int64_t j0 = (int64_t)blockIdx.y * per, j1 = min(n, j0 + per);
    double acc = 0.0;
    for (int64_t j = j0; j < j1; ++j) {
        double r2 = 0.0;
#pragma unroll
        for (int d = 0; d < D; ++d) {
            double diff = (double)Y[j * D + d] - xi[d];
            r2 = fma(diff, diff, r2);
        }
        acc = fma(exp(r2 * nc), (double)b[j], acc);
    }
    if (active) part[(int64_t)blockIdx.y * m + a] = acc;
}
__global__ __launch_bounds__(256) void rows_f64_sum_kernel(const double *__restrict__ part, int64_t m, int slices,
                                                           double *__restrict__ y64) {
    int64_t a = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (a >= m) return;
    double s = 0.0;
    for (int k = 0; k < slices; ++k) s += part[(int64_t)k * m + a];
    y64[a] = s;
}

// ------------------------------------------------------------------------------------
// tensor-product Lagrange weights of one point of a box: for each dimension the local
// coordinate t = (x - centre) / (l/2) is formed in fp64 (centre = alpha + (c + 1/2) l), the
// p basis values in fp32 by the product form.  out[d*p + i] = L_i(t_d).
// ------------------------------------------------------------------------------------
template <int D>
__device__ inline void point_weights(const float *__restrict__ x, const int32_t *__restrict__ cell,
                                     const CentreArg &C, const NodeArg &N, int p, float *out) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
        double centre = C.alpha[d] + ((double)cell[d] + 0.5) * C.edge;
        float t = (float)(((double)x[d] - centre) * C.inv_half);
        for (int i = 0; i < p; ++i) {
            float num = 1.f;
            for (int j = 0; j < p; ++j)
                if (j != i) num *= t - N.s[j];
            out[d * p + i] = num * N.invden[i];
        }
    }
}

// node index -> packed digits (4 bits per dimension)
template <int D>
__device__ inline uint32_t node_code(int i, int p) {
    uint32_t code = 0;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        code |= (uint32_t)(i % p) << (4 * d);
        i /= p;
    }
    return code;
}

// ------------------------------------------------------------------------------------
// P2M, v1 = L_Y b (Fig. 4 step 1): W_q[i] = sum_{j in q} L_i(t_j) b_j.
// One block per chunk (a run of <= P2M_CHUNK points of one box), one thread per node (or
// several nodes per thread when r > NT); points are staged 64 at a time through LDS as
// their 1-D basis values.  No atomics: a box with several chunks gets partial sums that
// p2m_reduce_kernel adds in a fixed order.
// ------------------------------------------------------------------------------------
constexpr int FF_TP = 64;  // points staged per step

template <int D, int NT>
__global__ __launch_bounds__(NT) void p2m_kernel(const float *__restrict__ Xs, const float *__restrict__ bs,
                                                 const uint32_t *__restrict__ start, const int32_t *__restrict__ cell,
                                                 const uint32_t *__restrict__ chunk_box,
                                                 const uint32_t *__restrict__ chunk_first, int64_t nchunks, int p,
                                                 int r, CentreArg C, NodeArg N, float *__restrict__ W,
                                                 float *__restrict__ Wpart) {
    constexpr int NPT_MAX = NT == 64 ? 1 : MAX_NODES / 256;
    extern __shared__ float lds[];
    const int DP = D * p;
    float *wts = lds;                 // [FF_TP][DP]
    float *bj = lds + FF_TP * DP;     // [FF_TP]
    const int64_t c = block_index();
    if (c >= nchunks) return;
    const uint32_t a = chunk_box[c];
    const uint32_t ci = (uint32_t)(c - chunk_first[a]);
    const uint32_t nch = chunk_first[a + 1] - chunk_first[a];
    const uint32_t k0 = start[a] + ci * (uint32_t)P2M_CHUNK;
    const uint32_t k1 = min(k0 + (uint32_t)P2M_CHUNK, start[a + 1]);
    const int npt = (r + NT - 1) / NT;
    uint32_t code[NPT_MAX];
    float acc[NPT_MAX];
#pragma unroll
    for (int m = 0; m < NPT_MAX; ++m) {
        int i = threadIdx.x + m * NT;
        code[m] = node_code<D>(i < r ? i : 0, p);
        acc[m] = 0.f;
    }
    for (uint32_t kb = k0; kb < k1; kb += FF_TP) {
        const int cnt = (int)min((uint32_t)FF_TP, k1 - kb);
        __syncthreads();
        if ((int)threadIdx.x < cnt) {
            const int64_t k = (int64_t)kb + threadIdx.x;
            point_weights<D>(Xs + k * D, cell + (int64_t)a * D, C, N, p, wts + threadIdx.x * DP);
            bj[threadIdx.x] = bs[k];
        }
        __syncthreads();
        for (int jj = 0; jj < cnt; ++jj) {
            const float *wj = wts + jj * DP;
            const float bv = bj[jj];
#pragma unroll
            for (int m = 0; m < NPT_MAX; ++m) {
                if (m < npt) {
                    float prod = bv;
#pragma unroll
                    for (int d = 0; d < D; ++d) prod *= wj[d * p + ((code[m] >> (4 * d)) & 15u)];
                    acc[m] += prod;
                }
            }
        }
    }
    float *dst = nch == 1 ? W + (int64_t)a * r : Wpart + c * r;
#pragma unroll
    for (int m = 0; m < NPT_MAX; ++m) {
        int i = threadIdx.x + m * NT;
        if (m < npt && i < r) dst[i] = acc[m];
    }
}

// boxes that were split into several chunks: add the partial node weights, chunk by
// chunk in ascending order, in fp64
__global__ __launch_bounds__(256) void p2m_reduce_kernel(const uint32_t *__restrict__ chunk_first, int64_t nb, int r,
                                                         const float *__restrict__ Wpart, float *__restrict__ W) {
    const int64_t a = block_index();
    if (a >= nb) return;
    const uint32_t c0 = chunk_first[a], c1 = chunk_first[a + 1];
    if (c1 - c0 <= 1) return;
    __shared__ double part[4][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    for (int i0 = 0; i0 < r; i0 += 64) {
        const int i = i0 + lane;
        double s = 0.0;
        if (i < r)
            for (uint32_t c = c0 + g; c < c1; c += 4) s += (double)Wpart[(int64_t)c * r + i];
        __syncthreads();
        part[g][lane] = s;
        __syncthreads();
        if (g == 0 && i < r) W[(int64_t)a * r + i] = (float)(((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane]);
    }
}

// Two-stage form for boxes with very many chunks: a block adds the partial node weights of one
// slice (at most P2M_SLICE chunks of one box) in fp64, then a block per box adds its slices,
// both in a fixed order.
__global__ __launch_bounds__(256) void p2m_slice_kernel(const uint32_t *__restrict__ slice_box,
                                                        const uint32_t *__restrict__ slice_first,
                                                        const uint32_t *__restrict__ chunk_first, int64_t nslices, int r,
                                                        const float *__restrict__ Wpart, double *__restrict__ Wslice) {
    const int64_t sidx = block_index();
    if (sidx >= nslices) return;
    const uint32_t a = slice_box[sidx];
    const uint32_t c0 = chunk_first[a] + (uint32_t)(sidx - slice_first[a]) * (uint32_t)P2M_SLICE;
    const uint32_t c1 = min(c0 + (uint32_t)P2M_SLICE, chunk_first[a + 1]);
    __shared__ double part[4][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    for (int i0 = 0; i0 < r; i0 += 64) {
        const int i = i0 + lane;
        double s = 0.0;
        if (i < r)
            for (uint32_t c = c0 + g; c < c1; c += 4) s += (double)Wpart[(int64_t)c * r + i];
        __syncthreads();
        part[g][lane] = s;
        __syncthreads();
        if (g == 0 && i < r) Wslice[sidx * r + i] = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
    }
}
__global__ __launch_bounds__(256) void p2m_slice_sum_kernel(const uint32_t *__restrict__ slice_first,
                                                            const uint32_t *__restrict__ chunk_first, int64_t nb, int r,
                                                            const double *__restrict__ Wslice, float *__restrict__ W) {
    const int64_t a = block_index();
    if (a >= nb) return;
    if (chunk_first[a + 1] - chunk_first[a] <= 1) return;   // the P2M kernel wrote W itself
    const uint32_t s0 = slice_first[a], s1 = slice_first[a + 1];
    for (int i = threadIdx.x; i < r; i += 256) {
        double s = 0.0;
        for (uint32_t k = s0; k < s1; ++k) s += Wslice[(int64_t)k * r + i];
        W[(int64_t)a * r + i] = (float)s;
    }
}

// ------------------------------------------------------------------------------------
// L2P, v = L_X^T v2 (Fig. 4 step 3): y_a += sum_i L_i(t_a) V_p[i] for the points a of box p.
// One block per chunk, one thread per point; V_p and the 1-D basis values sit in LDS.
// ------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(P2M_CHUNK) void l2p_kernel(const float *__restrict__ Xs,
                                                        const uint32_t *__restrict__ start,
                                                        const int32_t *__restrict__ cell,
                                                        const uint64_t *__restrict__ far_ptr,
                                                        const uint32_t *__restrict__ chunk_box,
                                                        const uint32_t *__restrict__ chunk_first, int64_t nchunks,
                                                        int p, int r, CentreArg C, NodeArg N,
                                                        const float *__restrict__ V, float *__restrict__ ys) {
    extern __shared__ float lds[];
    const int DP = D * p, stride = DP + 1;
    float *Vs = lds;          // [r]
    float *wts = lds + r;     // [P2M_CHUNK][stride]
    const int64_t c = block_index();
    if (c >= nchunks) return;
    const uint32_t a = chunk_box[c];
    if (far_ptr[a + 1] == far_ptr[a]) return;  // no far partner at this depth: V_p is zero
    const uint32_t ci = (uint32_t)(c - chunk_first[a]);
    const uint32_t k = start[a] + ci * (uint32_t)P2M_CHUNK + threadIdx.x;
    const bool active = k < start[a + 1];
    for (int i = threadIdx.x; i < r; i += P2M_CHUNK) Vs[i] = V[(int64_t)a * r + i];
    float *w = wts + threadIdx.x * stride;
    if (active) point_weights<D>(Xs + (int64_t)k * D, cell + (int64_t)a * D, C, N, p, w);
    __syncthreads();
    if (!active) return;
    int dig[D];
#pragma unroll
    for (int d = 0; d < D; ++d) dig[d] = 0;
    float acc = 0.f;
    for (int i = 0; i < r; ++i) {
        float prod = Vs[i];
#pragma unroll
        for (int d = 0; d < D; ++d) prod *= w[d * p + dig[d]];
        acc += prod;
        // next multi-index, dimension 0 fastest
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (++dig[d] < p) break;
            dig[d] = 0;
        }
    }
    ys[k] += acc;
}

// ------------------------------------------------------------------------------------
// P2M and L2P for D = 3 with 4 nodes per dimension (r = 64 = one wavefront): one wave per
// chunk, one lane per POINT.  The nodes are {1, 1/2, -1/2, -1}; the product-form basis of one
// coordinate costs 4 subtractions and 10 multiplications.
//   P2M: every lane keeps all 64 node sums of its own points in registers (64 FMAs per point
//        after 20 multiplications for the partial products), and the 64 x 64 lane-by-node
//        array is summed over lanes once per chunk through LDS (lane i ends up with node i).
//   L2P: V of the box is wave-uniform (scalar operands); the tensor contraction is nested:
//        64 + 16 + 4 FMAs per point.
// ------------------------------------------------------------------------------------
__device__ inline void lagrange4(float t, float (&L)[4]) {
    const float d0 = t - 1.f, d1 = t - 0.5f, d2 = t + 0.5f, d3 = t + 1.f;
    const float p01 = d0 * d1, p23 = d2 * d3;
    L[0] = d1 * p23 * (1.f / 1.5f);
    L[1] = d0 * p23 * (-1.f / 0.75f);
    L[2] = p01 * d3 * (1.f / 0.75f);
    L[3] = p01 * d2 * (-1.f / 1.5f);
}

__device__ inline void weights34(const float *__restrict__ x, const double (&ctr)[3], double inv_half, float (&Lx)[4],
                                 float (&Ly)[4], float (&Lz)[4]) {
    lagrange4((float)(((double)x[0] - ctr[0]) * inv_half), Lx);
    lagrange4((float)(((double)x[1] - ctr[1]) * inv_half), Ly);
    lagrange4((float)(((double)x[2] - ctr[2]) * inv_half), Lz);
}

constexpr int TR_STRIDE = 36;  // floats per lane row in the LDS transpose of 32 accumulators (16-byte aligned, bank-shifted)
constexpr int P2M_NCH = 4;     // chunks per wavefront: the table reads and the first loads of all of them are in
                               // flight together (a chunk alone is a chain of dependent loads, and the kernel was
                               // bound by that latency)

__global__ __launch_bounds__(64) void p2m34_kernel(const float *__restrict__ Xs, const float *__restrict__ bs,
                                                   const uint32_t *__restrict__ start, const int32_t *__restrict__ cell,
                                                   const uint32_t *__restrict__ chunk_box,
                                                   const uint32_t *__restrict__ chunk_first, int64_t nchunks, CentreArg C,
                                                   float *__restrict__ W, float *__restrict__ Wpart, int one_chunk) {
    // one_chunk: every box is a single chunk (chunk index = box rank): two dependent table reads less
    __shared__ float tr[64 * TR_STRIDE];
    const int64_t c0 = block_index() * P2M_NCH;
    if (c0 >= nchunks) return;
    const int lane = threadIdx.x;
    // chunk j of this wavefront (a chunk beyond the end repeats the last one and is switched off)
    uint32_t a[P2M_NCH], k0[P2M_NCH], k1[P2M_NCH], nch[P2M_NCH];
    int64_t cj[P2M_NCH];
    bool on[P2M_NCH];
#pragma unroll
    for (int j = 0; j < P2M_NCH; ++j) {
        cj[j] = c0 + j < nchunks ? c0 + j : nchunks - 1;
        on[j] = c0 + j < nchunks;
        a[j] = one_chunk ? (uint32_t)cj[j] : (uint32_t)__builtin_amdgcn_readfirstlane(chunk_box[cj[j]]);
    }
    double ctr[P2M_NCH][3];
#pragma unroll
    for (int j = 0; j < P2M_NCH; ++j) {
        const uint32_t ci = one_chunk ? 0u : (uint32_t)(cj[j] - chunk_first[a[j]]);
        nch[j] = one_chunk ? 1u : chunk_first[a[j] + 1] - chunk_first[a[j]];
        k0[j] = start[a[j]] + ci * (uint32_t)P2M_CHUNK;     // a point of the box: always a valid index
        k1[j] = min(k0[j] + (uint32_t)P2M_CHUNK, start[a[j] + 1]);
#pragma unroll
        for (int d = 0; d < 3; ++d) ctr[j][d] = C.alpha[d] + ((double)cell[(int64_t)a[j] * 3 + d] + 0.5) * C.edge;
    }
    // Loads are unconditional, the index of a lane beyond the chunk clamped to the chunk's first point
    // and its weight set to zero (a branch around them would make every load wait on its own).
    auto load = [&](int j, uint32_t kb, float (&x)[3], float &bv) {
        const uint32_t k = kb + lane;
        const bool live = k < k1[j];
        const uint32_t kc = live ? k : k0[j];
#pragma unroll
        for (int d = 0; d < 3; ++d) x[d] = Xs[(int64_t)kc * 3 + d];
        const float bl = bs[kc];
        bv = live ? bl : 0.f;
    };
    float x[P2M_NCH][3], bv[P2M_NCH];
#pragma unroll
    for (int j = 0; j < P2M_NCH; ++j) load(j, k0[j], x[j], bv[j]);
    const int i = lane & 31, part = lane >> 5;
#pragma unroll
    for (int j = 0; j < P2M_NCH; ++j) {
        if (!on[j]) continue;   // wave-uniform
        float acc[64];
#pragma unroll
        for (int q = 0; q < 64; ++q) acc[q] = 0.f;
        float xc[3] = {x[j][0], x[j][1], x[j][2]}, bc = bv[j];
        for (uint32_t kb = k0[j];;) {
            // the next run of the chunk (boxes above 64 points) is loaded while this one is added
            const bool more = kb + 64 < k1[j];
            float xn[3] = {0.f, 0.f, 0.f}, bn = 0.f;
            if (more) load(j, kb + 64, xn, bn);
            float Lx[4], Ly[4], Lz[4];
            weights34(xc, ctr[j], C.inv_half, Lx, Ly, Lz);
#pragma unroll
            for (int i3 = 0; i3 < 4; ++i3) {
                const float zb = Lz[i3] * bc;
#pragma unroll
                for (int i2 = 0; i2 < 4; ++i2) {
                    const float yz = Ly[i2] * zb;
#pragma unroll
                    for (int i1 = 0; i1 < 4; ++i1) acc[i1 + 4 * i2 + 16 * i3] = fmaf(Lx[i1], yz, acc[i1 + 4 * i2 + 16 * i3]);
                }
            }
            if (!more) break;
            kb += 64;
#pragma unroll
            for (int d = 0; d < 3; ++d) xc[d] = xn[d];
            bc = bn;
        }
        // sum over lanes, 32 nodes at a time (half the LDS, twice the resident wavefronts): lane l
        // writes its row; lane (i, part) adds rows 32 part .. 32 part + 31 of column i, and the two
        // parts meet through one shuffle
        float *dst = nch[j] == 1 ? W + (int64_t)a[j] * 64 : Wpart + cj[j] * 64;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            __syncthreads();   // the sums of the previous half (or chunk) have been read
#pragma unroll
            for (int g = 0; g < 8; ++g)
                *reinterpret_cast<float4 *>(&tr[lane * TR_STRIDE + 4 * g]) =
                    make_float4(acc[32 * q + 4 * g], acc[32 * q + 4 * g + 1], acc[32 * q + 4 * g + 2], acc[32 * q + 4 * g + 3]);
            __syncthreads();
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
            for (int row = 0; row < 32; row += 4) {
                s0 += tr[(32 * part + row + 0) * TR_STRIDE + i];
                s1 += tr[(32 * part + row + 1) * TR_STRIDE + i];
                s2 += tr[(32 * part + row + 2) * TR_STRIDE + i];
                s3 += tr[(32 * part + row + 3) * TR_STRIDE + i];
            }
            float t = (s0 + s1) + (s2 + s3);
            t += __shfl_xor(t, 32, 64);
            if (part == 0) dst[32 * q + i] = t;
        }
    }
}

// P2M where every box is one chunk (no box above P2M_CHUNK points): a box per HALF wavefront.  The kernel is
// bound by its instruction stream, and a third of that stream is the sum of the 64 accumulators over the lanes;
// with 32 lanes per box that sum covers two boxes at once (per pass of 32 accumulators a lane adds 32 rows
// instead of 32 rows of one box out of 64), and a box of some 60 points takes two rounds of 32 lanes instead of
// one round of 64, which costs the same.  Lane = point; the two halves of a wavefront work on boxes a and a + 1,
// four such pairs per wavefront with the first loads of all of them in flight together.
constexpr int P2M_NPAIR = 4;
__global__ __launch_bounds__(64) void p2m34_pair_kernel(const float *__restrict__ Xs, const float *__restrict__ bs,
                                                        const uint32_t *__restrict__ start,
                                                        const int32_t *__restrict__ cell, int64_t nb, CentreArg C,
                                                        float *__restrict__ W) {
    // rows of the upper half are shifted by 32 floats so that the two halves read different banks
    __shared__ __attribute__((aligned(16))) float tr[64 * TR_STRIDE + 32];
    const int64_t b0 = block_index() * (2 * P2M_NPAIR);
    if (b0 >= nb) return;
    const int lane = threadIdx.x, half = lane >> 5, t = lane & 31;
    uint32_t k0[P2M_NPAIR], k1[P2M_NPAIR];
    int64_t a[P2M_NPAIR];
    bool on[P2M_NPAIR];
    double ctr[P2M_NPAIR][3];
#pragma unroll
    for (int j = 0; j < P2M_NPAIR; ++j) {
        a[j] = b0 + 2 * j + half;
        on[j] = a[j] < nb;
        const int64_t ac = on[j] ? a[j] : nb - 1;
        k0[j] = start[ac];
        k1[j] = on[j] ? start[ac + 1] : k0[j];   // a box beyond the end has no points
#pragma unroll
        for (int d = 0; d < 3; ++d) ctr[j][d] = C.alpha[d] + ((double)cell[ac * 3 + d] + 0.5) * C.edge;
    }
    // Loads are unconditional, the index of a lane beyond the box clamped to the box's first point and its
    // weight set to zero (a branch around them would make every load wait on its own).
    auto load = [&](int j, uint32_t kb, float (&x)[3], float &bv) __attribute__((always_inline)) {
        const uint32_t k = kb + (uint32_t)t;
        const bool live = k < k1[j];
        const uint32_t kc = live ? k : k0[j];
#pragma unroll
        for (int d = 0; d < 3; ++d) x[d] = Xs[(int64_t)kc * 3 + d];
        const float bl = bs[kc];
        bv = live ? bl : 0.f;
    };
    float x[P2M_NPAIR][3], bv[P2M_NPAIR];
#pragma unroll
    for (int j = 0; j < P2M_NPAIR; ++j) load(j, k0[j], x[j], bv[j]);
    const int rowbase = lane * TR_STRIDE + half * 32;
#pragma unroll
    for (int j = 0; j < P2M_NPAIR; ++j) {
        if (b0 + 2 * j >= nb) break;   // wave-uniform: neither box of the pair exists
        float acc[64];
#pragma unroll
        for (int q = 0; q < 64; ++q) acc[q] = 0.f;
        float xc[3] = {x[j][0], x[j][1], x[j][2]}, bc = bv[j];
        for (uint32_t kb = k0[j];;) {
            // the next round (a box above 32 points) is loaded while this one is added; the wavefront goes on
            // while either half has points left
            const bool more = __ballot(kb + 32 < k1[j]) != 0ull;
            float xn[3] = {0.f, 0.f, 0.f}, bn = 0.f;
            if (more) load(j, kb + 32, xn, bn);
            float Lx[4], Ly[4], Lz[4];
            weights34(xc, ctr[j], C.inv_half, Lx, Ly, Lz);
#pragma unroll
            for (int i3 = 0; i3 < 4; ++i3) {
                const float zb = Lz[i3] * bc;
#pragma unroll
                for (int i2 = 0; i2 < 4; ++i2) {
                    const float yz = Ly[i2] * zb;
#pragma unroll
                    for (int i1 = 0; i1 < 4; ++i1) acc[i1 + 4 * i2 + 16 * i3] = fmaf(Lx[i1], yz, acc[i1 + 4 * i2 + 16 * i3]);
                }
            }
            if (!more) break;
            kb += 32;
#pragma unroll
            for (int d = 0; d < 3; ++d) xc[d] = xn[d];
            bc = bn;
        }
        // sum over the 32 lanes of each half, 32 nodes at a time: lane l writes its row; lane t of a half adds
        // the 32 rows of its half in column t
        float *dst = W + a[j] * 64;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            __syncthreads();   // the sums of the previous pass (or pair) have been read
#pragma unroll
            for (int g = 0; g < 8; ++g)
                *reinterpret_cast<float4 *>(&tr[rowbase + 4 * g]) =
                    make_float4(acc[32 * q + 4 * g], acc[32 * q + 4 * g + 1], acc[32 * q + 4 * g + 2], acc[32 * q + 4 * g + 3]);
            __syncthreads();
            const float *col = tr + (32 * half) * TR_STRIDE + half * 32 + t;
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
            for (int row = 0; row < 32; row += 4) {
                s0 += col[(row + 0) * TR_STRIDE];
                s1 += col[(row + 1) * TR_STRIDE];
                s2 += col[(row + 2) * TR_STRIDE];
                s3 += col[(row + 3) * TR_STRIDE];
            }
            if (on[j]) dst[32 * q + t] = (s0 + s1) + (s2 + s3);
        }
    }
}

constexpr int L2P_NCH = 4;   // chunks per wavefront: their loads are in flight together (a chunk alone is a chain
                             // of dependent loads and the kernel is bound by that latency)
__global__ __launch_bounds__(64) void l2p34_kernel(const float *__restrict__ Xs, const uint32_t *__restrict__ start,
                                                   const int32_t *__restrict__ cell,
                                                   const uint64_t *__restrict__ far_ptr,
                                                   const uint32_t *__restrict__ chunk_box,
                                                   const uint32_t *__restrict__ chunk_first, int64_t nchunks, CentreArg C,
                                                   const float *__restrict__ V, float *__restrict__ ys, int one_chunk) {
    // one_chunk: every box is a single chunk (chunk index = box rank): two dependent table reads less
    __shared__ __attribute__((aligned(16))) float vbuf[L2P_NCH][64];
    const int64_t c0 = block_index() * L2P_NCH;
    if (c0 >= nchunks) return;
    const int lane = threadIdx.x;
    // chunk j of this wavefront (a chunk beyond the end repeats the last one and is switched off)
    uint32_t a[L2P_NCH], k0[L2P_NCH], k1[L2P_NCH];
    bool on[L2P_NCH];
#pragma unroll
    for (int j = 0; j < L2P_NCH; ++j) {
        const int64_t c = c0 + j < nchunks ? c0 + j : nchunks - 1;
        on[j] = c0 + j < nchunks;
        a[j] = one_chunk ? (uint32_t)c : (uint32_t)__builtin_amdgcn_readfirstlane(chunk_box[c]);
    }
    double ctr[L2P_NCH][3];
    float vrow[L2P_NCH];
#pragma unroll
    for (int j = 0; j < L2P_NCH; ++j) {
        const int64_t c = c0 + j < nchunks ? c0 + j : nchunks - 1;
        // far_ptr given: skip boxes without far partner at this depth (V_p is zero); nullptr: V holds the
        // potentials accumulated over all depths and every box is evaluated
        if (far_ptr && far_ptr[a[j] + 1] == far_ptr[a[j]]) on[j] = false;
        const uint32_t ci = one_chunk ? 0u : (uint32_t)(c - chunk_first[a[j]]);
        k0[j] = start[a[j]] + ci * (uint32_t)P2M_CHUNK;     // a point of the box: always a valid index
        k1[j] = min(k0[j] + (uint32_t)P2M_CHUNK, start[a[j] + 1]);
        if (!on[j]) k1[j] = k0[j];
#pragma unroll
        for (int d = 0; d < 3; ++d) ctr[j][d] = C.alpha[d] + ((double)cell[(int64_t)a[j] * 3 + d] + 0.5) * C.edge;
        vrow[j] = V[(int64_t)a[j] * 64 + lane];             // the node potentials of the box, one per lane
    }
    // The node potentials reach the lanes as LDS broadcasts (every lane reads the same address);
    // as scalar operands they arrive in four dependent batches per box.
#pragma unroll
    for (int j = 0; j < L2P_NCH; ++j) vbuf[j][lane] = vrow[j];
    __builtin_amdgcn_wave_barrier();   // one wavefront per block; its LDS operations complete in order
    // one run of 64 points of a chunk: y += sum_i L_i(t) V[i], nested over the dimensions
    auto run = [&](int j, bool live, uint32_t k, const float (&x)[3], float yold) {
        float Lx[4], Ly[4], Lz[4];
        weights34(x, ctr[j], C.inv_half, Lx, Ly, Lz);
        float y = 0.f;
#pragma unroll
        for (int i3 = 0; i3 < 4; ++i3) {
            float sy = 0.f;
#pragma unroll
            for (int i2 = 0; i2 < 4; ++i2) {
                const float4 v = *reinterpret_cast<const float4 *>(&vbuf[j][4 * i2 + 16 * i3]);
                float sx = Lx[0] * v.x;
                sx = fmaf(Lx[1], v.y, sx);
                sx = fmaf(Lx[2], v.z, sx);
                sx = fmaf(Lx[3], v.w, sx);
                sy = fmaf(Ly[i2], sx, sy);
            }
            y = fmaf(Lz[i3], sy, y);
        }
        if (live) ys[k] = yold + y;
    };
    // Loads are unconditional with the index of a lane beyond the chunk clamped to the chunk's first
    // point (a branch around them would make the compiler wait for every load on its own); the first
    // run of every chunk has all its loads issued before any is used, then what is left of the chunks.
    float x[L2P_NCH][3], yold[L2P_NCH];
    bool live[L2P_NCH];
    uint32_t kk[L2P_NCH];
#pragma unroll
    for (int j = 0; j < L2P_NCH; ++j) {
        const uint32_t k = k0[j] + lane;
        live[j] = k < k1[j];
        kk[j] = live[j] ? k : k0[j];
#pragma unroll
        for (int d = 0; d < 3; ++d) x[j][d] = Xs[(int64_t)kk[j] * 3 + d];
        yold[j] = ys[kk[j]];
    }
#pragma unroll
    for (int j = 0; j < L2P_NCH; ++j) run(j, live[j], kk[j], x[j], yold[j]);
#pragma unroll
    for (int j = 0; j < L2P_NCH; ++j) {
        for (uint32_t kb = k0[j] + 64; kb < k1[j]; kb += 64) {
            const uint32_t k = kb + lane;
            const bool lv = k < k1[j];
            const uint32_t kc = lv ? k : k0[j];
            float xr[3];
#pragma unroll
            for (int d = 0; d < 3; ++d) xr[d] = Xs[(int64_t)kc * 3 + d];
            run(j, lv, kc, xr, ys[kc]);
        }
    }
}

// ------------------------------------------------------------------------------------
// Node weights and node potentials between depths (D = 3, 4 nodes per dimension).
// The basis functions of a parent box are polynomials of degree 3 per coordinate, and the
// 4-node interpolant of a child box reproduces such polynomials exactly.  Hence
//   W_parent[i] = sum_children sum_k L^parent_i(s^child_k) W_child[k]           (upward)
// equals the P2M sum over the parent's points, and evaluating a parent's potential at a
// child's nodes,  V_child[k] += sum_i L^parent_i(s^child_k) V_parent[i]          (downward),
// followed by ONE L2P at the last depth equals the per-depth L2P sums -- both up to
// rounding.  This replaces the streaming passes over all points at every depth (Fig. 4
// steps 1 and 3 per depth) by one pass each at the last depth.
// In parent coordinates the child's node k sits at (s_k -+ 1)/2 (lower / upper half), so the
// 64 x 64 transfer matrix is a tensor product of three 4 x 4 matrices T1[half][i][k].
// ------------------------------------------------------------------------------------
struct TransferArg { float t[2][4][4]; };   // t[half][i][k] = L_i((s_k + (half ? 1 : -1)) / 2)

static TransferArg make_transfer() {
    TransferArg T{};
    double s[4];
    for (int i = 0; i < 4; ++i) s[i] = std::cos((double)i * M_PI / 3.0);
    for (int h = 0; h < 2; ++h)
        for (int k = 0; k < 4; ++k) {
            const double tp = 0.5 * (s[k] + (h ? 1.0 : -1.0));
            for (int i = 0; i < 4; ++i) {
                double num = 1.0, den = 1.0;
                for (int j = 0; j < 4; ++j)
                    if (j != i) { num *= tp - s[j]; den *= s[i] - s[j]; }
                T.t[h][i][k] = (float)(num / den);
            }
        }
    return T;
}

void upload_transfer(f3m_plan_s &P, hipStream_t st) {
    const TransferArg T = make_transfer();
    P.transfer.alloc(32, &P.bytes);
    F3M_HIP(hipMemcpyAsync(P.transfer.p, &T.t[0][0][0], 32 * sizeof(float), hipMemcpyHostToDevice, st));
    F3M_HIP(hipStreamSynchronize(st));
}

// Both transfers run one wavefront per PARENT with lane = node (ix + 4 iy + 16 iz) and apply the
// three 4 x 4 factors one dimension at a time, 4 multiply-adds each: the other three entries of a
// fibre sit in the lane's quad (x: DPP quad permutations), in its row of 16 lanes (y: DPP row
// rotations by 4, 8, 12) and in the other rows (z: ds_bpermute).  f[k] is the factor entry for the
// fibre element k places further on (cyclically).  All rows of the (at most 8) children are loaded
// before the first is used: one round of memory latency per parent.
template <int CTRL>
__device__ inline float dpp_take(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

__device__ inline float fibre_x(float v, const float (&f)[4]) {
    float o = f[0] * v;
    o = fmaf(f[1], dpp_take<0x39>(v), o);    // quad_perm [1,2,3,0]
    o = fmaf(f[2], dpp_take<0x4E>(v), o);    // quad_perm [2,3,0,1]
    return fmaf(f[3], dpp_take<0x93>(v), o); // quad_perm [3,0,1,2]
}

__device__ inline float fibre_y(float v, const float (&f)[4]) {
    float o = f[0] * v;
    o = fmaf(f[1], dpp_take<0x12C>(v), o);    // row_ror:12 = the lane 4 further on in the row of 16
    o = fmaf(f[2], dpp_take<0x128>(v), o);    // row_ror:8
    return fmaf(f[3], dpp_take<0x124>(v), o); // row_ror:4
}

__device__ inline float fibre_z(float v, const float (&f)[4], int lane) {
    float o = f[0] * v;
#pragma unroll
    for (int k = 1; k < 4; ++k) o = fmaf(f[k], __shfl(v, (lane + 16 * k) & 63, 64), o);
    return o;
}

// W_parent[i] = sum over children, sum_k T[half][i][k] (per dimension) W_child[k]
__global__ __launch_bounds__(64) void m2m34_kernel(const uint32_t *__restrict__ cstart,
                                                   const uint32_t *__restrict__ child_key, int64_t nparents,
                                                   const float *__restrict__ T, const float *__restrict__ Wchild,
                                                   float *__restrict__ Wparent) {
    __shared__ float tl[32];
    const int64_t P = block_index();
    if (P >= nparents) return;
    const int lane = threadIdx.x, ix = lane & 3, iy = (lane >> 2) & 3, iz = lane >> 4;
    const uint32_t c0 = cstart[P];
    const int nc = min((int)(cstart[P + 1] - c0), 8);   // a box has at most 2^3 children
    if (nc <= 0) {                                      // (boxes are never empty: cannot happen)
        Wparent[P * 64 + lane] = 0.f;
        return;
    }
    if (lane < 32) tl[lane] = T[lane];
    const uint32_t key = child_key[c0 + (uint32_t)min(lane, nc - 1)];
    float w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) w[j] = Wchild[(int64_t)(c0 + (uint32_t)min(j, nc - 1)) * 64 + lane];
    __syncthreads();
    float f[3][2][4];   // [dimension][half][k]: T[half][i][(i + k) & 3] with i the lane's node index in that dimension
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[0][h][k] = tl[h * 16 + ix * 4 + ((ix + k) & 3)];
            f[1][h][k] = tl[h * 16 + iy * 4 + ((iy + k) & 3)];
            f[2][h][k] = tl[h * 16 + iz * 4 + ((iz + k) & 3)];
        }
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (j < nc) {
            const uint32_t par = (uint32_t)__builtin_amdgcn_readlane((int)key, j) & 7u;   // bit d = upper half along d
            float g[3][4];
#pragma unroll
            for (int d = 0; d < 3; ++d)
#pragma unroll
                for (int k = 0; k < 4; ++k) g[d][k] = (par >> d) & 1u ? f[d][1][k] : f[d][0][k];
            acc += fibre_z(fibre_y(fibre_x(w[j], g[0]), g[1]), g[2], lane);
        }
    }
    Wparent[P * 64 + lane] = acc;
}

// V_child[k] += sum_i T[half][i][k] (per dimension) V_parent[i], for every child of the parent
__global__ __launch_bounds__(64) void l2l34_kernel(const uint32_t *__restrict__ cstart,
                                                   const uint32_t *__restrict__ child_key, int64_t nparents,
                                                   const float *__restrict__ T, const float *__restrict__ Vparent,
                                                   float *__restrict__ Vchild) {
    __shared__ float tl[32];
    const int64_t P = block_index();
    if (P >= nparents) return;
    const int lane = threadIdx.x, kx = lane & 3, ky = (lane >> 2) & 3, kz = lane >> 4;
    const uint32_t c0 = cstart[P];
    const int nc = min((int)(cstart[P + 1] - c0), 8);
    if (nc <= 0) return;
    if (lane < 32) tl[lane] = T[lane];
    const uint32_t key = child_key[c0 + (uint32_t)min(lane, nc - 1)];
    const float vp = Vparent[P * 64 + lane];
    float vc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) vc[j] = Vchild[(int64_t)(c0 + (uint32_t)min(j, nc - 1)) * 64 + lane];
    __syncthreads();
    float f[3][2][4];   // [dimension][half][j]: T[half][(k + j) & 3][k] with k the lane's node index in that dimension
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[0][h][j] = tl[h * 16 + ((kx + j) & 3) * 4 + kx];
            f[1][h][j] = tl[h * 16 + ((ky + j) & 3) * 4 + ky];
            f[2][h][j] = tl[h * 16 + ((kz + j) & 3) * 4 + kz];
        }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (j < nc) {
            const uint32_t par = (uint32_t)__builtin_amdgcn_readlane((int)key, j) & 7u;
            float g[3][4];
#pragma unroll
            for (int d = 0; d < 3; ++d)
#pragma unroll
                for (int k = 0; k < 4; ++k) g[d][k] = (par >> d) & 1u ? f[d][1][k] : f[d][0][k];
            Vchild[(int64_t)(c0 + (uint32_t)j) * 64 + lane] = vc[j] + fibre_z(fibre_y(fibre_x(vp, g[0]), g[1]), g[2], lane);
        }
    }
}

// ------------------------------------------------------------------------------------
// M2L for any D and node count (Fig. 4 step 2), V_t += K(s^t, s^q) W_q over the far row of t.
// The Gaussian is a product over dimensions, and so is the tensor grid of nodes, hence the
// node-to-node matrix of a far pair with cell offset o is a Kronecker product,
//   K = G_{o_D} x ... x G_{o_1},   G_o[i][j] = exp(-(l/2)^2 (2 o + s_j - s_i)^2 / (2 gamma^2)),
// of p x p matrices that depend on the offset in one dimension only.  It is applied one
// dimension at a time (D passes of r p multiply-adds instead of r^2 kernel values): the same
// sums as the dense product, in another order.  The table G[o + omax][i][j] is built in fp64
// per depth at plan time.
// Boxes with more than 32 fibres (a fibre = the p entries along one dimension) take
// m2l_kron_grouped_kernel, which also nests the sum over the far partners over the dimensions;
// boxes with fewer take m2l_kron_small_kernel, several far pairs per wavefront.
// For two point sets the grids are shifted by u_d box edges in dimension d, so the factor of
// dimension d depends on o + u_d: the table is kept per dimension, G[d][o - omin_d][i][j] with
// G = exp(-(l/2)^2 (2 (o + u_d) + s_j - s_i)^2 / (2 gamma^2)), `no` offsets per dimension
// (cellT: cells of the target boxes, cellS: of the source boxes; u = 0 and equal tables for one set).
// ------------------------------------------------------------------------------------
struct KronShape {
    int omin[F3M_MAX_DIM];   // smallest tabulated offset (source cell - target cell) per dimension
    int no;                  // tabulated offsets per dimension
};

// ---- far rows in the order of the row-major cell index ------------------------------------------
// The grouped M2L below shares work between far partners whose cells differ in the leading dimensions
// only, so it wants the partners of a target ordered by (c_{D-1}, ..., c_1, c_0), most significant first:
// ascending row-major index beta = sum_d c_d 2^(depth d) (the box index of Sec. 4.2).  The far lists are
// stored ascending in the interleaved key; far_ord holds every row once more in beta order.  A row is
// sorted in pieces of at most FO_CH entries (bitonic network in LDS); the M2L is correct for any
// order, a piece boundary only costs it a few shared sums.
constexpr int FO_CH = 8192;    // 64 KB of keys: two workgroups per compute unit
constexpr int FO_NT = 512;
__global__ __launch_bounds__(FO_NT) void far_order_kernel(const uint64_t *__restrict__ far_ptr,
                                                         const uint32_t *__restrict__ far_col,
                                                         const int32_t *__restrict__ cellS, int D, int depth, int64_t nb,
                                                         uint32_t *__restrict__ far_ord) {
    __shared__ uint64_t key[FO_CH];
    const int64_t a = block_index();
    if (a >= nb) return;
    const int tid = threadIdx.x;
    const uint64_t e0 = far_ptr[a], e1 = far_ptr[a + 1];
    for (uint64_t c0 = e0; c0 < e1; c0 += FO_CH) {
        const int len = (int)(e1 - c0 < (uint64_t)FO_CH ? e1 - c0 : (uint64_t)FO_CH);
        int n2 = 2;
        while (n2 < len) n2 <<= 1;
        for (int i = tid; i < n2; i += FO_NT) {
            uint64_t k = ~0ull;
            if (i < len) {
                const uint32_t q = far_col[c0 + i];
                uint64_t beta = 0;
                for (int d = 0; d < D; ++d) beta |= (uint64_t)(uint32_t)cellS[(int64_t)q * D + d] << (depth * d);
                k = (beta << 32) | q;
            }
            key[i] = k;
        }
        __syncthreads();
        for (int k = 2; k <= n2; k <<= 1)
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int i = tid; i < n2; i += FO_NT) {
                    const int ixj = i ^ j;
                    if (ixj > i) {
                        const uint64_t x = key[i], y = key[ixj];
                        if ((x > y) == ((i & k) == 0)) {
                            key[i] = y;
                            key[ixj] = x;
                        }
                    }
                }
                __syncthreads();
            }
        for (int i = tid; i < len; i += FO_NT) far_ord[c0 + i] = (uint32_t)key[i];
        __syncthreads();
    }
}

constexpr int ipow_c(int p, int d) { return d <= 0 ? 1 : p * ipow_c(p, d - 1); }

// Grouped M2L: the far partners q of a target t are taken in the order of far_ord, and the sum
//   V_t = sum_q (G_{o_{D-1}(q)} x ... x G_{o_0(q)}) W_q
// is nested over the dimensions,
//   V_t = sum_{o_{D-1}} G_{o_{D-1}} [ sum_{o_{D-2}} G_{o_{D-2}} [ ... sum_{o_0} G_{o_0} W_q ] ]:
// level d keeps a partial sum S_d over the partners that agree in (o_{d+1}, ..., o_{D-1}); when the next
// partner differs in one of those, S_d is multiplied by the factor of dimension d+1 and added to S_{d+1}
// ("flush").  Every partner costs one factor (dimension 0, on data straight from global memory), every
// group of a level one more, instead of D factors per partner: the same sums as the dense products, in
// another order.  For partners in any other order the result is the same (more flushes).
// One workgroup of 256 threads per target; a thread owns up to NFL fibres of every dimension (a fibre =
// the p entries along one dimension) and keeps S_d of its fibres of dimension d in registers; a flush
// passes S_d through LDS (node layout) to the owners of the fibres of dimension d+1, alternating
// between two buffers so that one barrier per flush is enough.
template <int PN, int DD>
__global__ __launch_bounds__(256) void m2l_kron_grouped_kernel(const int32_t *__restrict__ cellT,
                                                               const int32_t *__restrict__ cellS,
                                                               const uint64_t *__restrict__ far_ptr,
                                                               const uint32_t *__restrict__ far_ord, int64_t nb,
                                                               const float *__restrict__ G, KronShape S,
                                                               const float *__restrict__ W, float *__restrict__ V) {
    constexpr int R = ipow_c(PN, DD), NFIB = R / PN, NFL = (NFIB + 255) / 256;
    __shared__ float buf[2][R];
    const int64_t a = block_index();
    if (a >= nb) return;
    const uint64_t e0 = far_ptr[a], e1 = far_ptr[a + 1];
    if (e0 == e1) return;   // no far partner at this depth: the row of V is left alone
    const int tid = threadIdx.x;
    float acc[DD][NFL][PN];
#pragma unroll
    for (int d = 0; d < DD; ++d)
#pragma unroll
        for (int k = 0; k < NFL; ++k)
#pragma unroll
            for (int i = 0; i < PN; ++i) acc[d][k][i] = 0.f;
    int ca[DD], prev[DD];
#pragma unroll
    for (int d = 0; d < DD; ++d) ca[d] = cellT[a * DD + d];
    // factor matrix of dimension d for a source cell coordinate (the index is clamped to the table:
    // every far pair lies inside it by construction)
    auto factor = [&](int d, int cs) __attribute__((always_inline)) {
        int k = cs - ca[d] - S.omin[d];
        k = k < 0 ? 0 : (k >= S.no ? S.no - 1 : k);
        return G + ((int64_t)d * S.no + k) * (PN * PN);
    };
    int flip = 0;
    // S_d, times the factor of dimension d+1 for source cell coordinate cs1, is added to S_{d+1}; S_d = 0
    auto flush = [&](auto dconst, int cs1) __attribute__((always_inline)) {
        constexpr int d = decltype(dconst)::value;
        constexpr int sd = ipow_c(PN, d), sd1 = sd * PN;
        float *B = buf[flip];
        flip ^= 1;
#pragma unroll
        for (int k = 0; k < NFL; ++k) {
            const int f = tid + 256 * k;
            if (f < NFIB) {
                const int hi = f / sd, base = hi * sd1 + (f - hi * sd);
#pragma unroll
                for (int j = 0; j < PN; ++j) {
                    B[base + j * sd] = acc[d][k][j];
                    acc[d][k][j] = 0.f;
                }
            }
        }
        __syncthreads();
        const float *__restrict__ g = factor(d + 1, cs1);
#pragma unroll
        for (int k = 0; k < NFL; ++k) {
            const int f = tid + 256 * k;
            if (f < NFIB) {
                const int hi = f / sd1, base = hi * sd1 * PN + (f - hi * sd1);
                float in[PN];
#pragma unroll
                for (int j = 0; j < PN; ++j) in[j] = B[base + j * sd1];
#pragma unroll
                for (int i = 0; i < PN; ++i) {
                    float t = acc[d + 1][k][i];
#pragma unroll
                    for (int j = 0; j < PN; ++j) t = fmaf(g[i * PN + j], in[j], t);
                    acc[d + 1][k][i] = t;
                }
            }
        }
    };
    // the levels below `upto` end their groups (upto = DD: all of them)
    auto flush_below = [&](int upto) __attribute__((always_inline)) {
        if constexpr (DD > 1) { if (upto > 0) flush(std::integral_constant<int, 0>{}, prev[1]); }
        if constexpr (DD > 2) { if (upto > 1) flush(std::integral_constant<int, 1>{}, prev[2]); }
        if constexpr (DD > 3) { if (upto > 2) flush(std::integral_constant<int, 2>{}, prev[3]); }
        if constexpr (DD > 4) { if (upto > 3) flush(std::integral_constant<int, 3>{}, prev[4]); }
        if constexpr (DD > 5) { if (upto > 4) flush(std::integral_constant<int, 4>{}, prev[5]); }
        if constexpr (DD > 6) { if (upto > 5) flush(std::integral_constant<int, 5>{}, prev[6]); }
    };
    // the fibres of dimension 0 of a partner's node weights: p consecutive floats each
    auto load = [&](uint32_t q, float (&w)[NFL][PN]) __attribute__((always_inline)) {
        const float *Wq = W + (int64_t)q * R;
#pragma unroll
        for (int k = 0; k < NFL; ++k) {
            const int f = tid + 256 * k;
#pragma unroll
            for (int j = 0; j < PN; ++j) w[k][j] = f < NFIB ? Wq[f * PN + j] : 0.f;
        }
    };
    float wn[NFL][PN];
    uint32_t qn = __builtin_amdgcn_readfirstlane(far_ord[e0]);
    load(qn, wn);
    for (uint64_t e = e0; e < e1; ++e) {
        const uint32_t q = qn;
        float wc[NFL][PN];
#pragma unroll
        for (int k = 0; k < NFL; ++k)
#pragma unroll
            for (int j = 0; j < PN; ++j) wc[k][j] = wn[k][j];
        if (e + 1 < e1) {   // the next partner's weights are on their way during this one's sums
            qn = __builtin_amdgcn_readfirstlane(far_ord[e + 1]);
            load(qn, wn);
        }
        int cs[DD];
#pragma unroll
        for (int d = 0; d < DD; ++d) cs[d] = __builtin_amdgcn_readfirstlane(cellS[(int64_t)q * DD + d]);
        if (e > e0) {
            int upto = 0;   // one more than the highest dimension >= 1 in which this partner differs from the last
#pragma unroll
            for (int d = 1; d < DD; ++d) upto = cs[d] != prev[d] ? d : upto;
            flush_below(upto);
        }
        const float *__restrict__ g = factor(0, cs[0]);
#pragma unroll
        for (int k = 0; k < NFL; ++k)
#pragma unroll
            for (int i = 0; i < PN; ++i) {
                float t = acc[0][k][i];
#pragma unroll
                for (int j = 0; j < PN; ++j) t = fmaf(g[i * PN + j], wc[k][j], t);
                acc[0][k][i] = t;
            }
#pragma unroll
        for (int d = 0; d < DD; ++d) prev[d] = cs[d];
    }
    flush_below(DD);
    // S_{D-1} is the row of V: node (fibre f of the last dimension, entry j) = j r/p + f
    float *Va = V + a * R;
#pragma unroll
    for (int k = 0; k < NFL; ++k) {
        const int f = tid + 256 * k;
        if (f < NFIB) {
#pragma unroll
            for (int j = 0; j < PN; ++j) Va[j * NFIB + f] = acc[DD - 1][k][j];
        }
    }
}

// The same for boxes with few fibres (r/p <= 32, e.g. D = 3 with 4 nodes per dimension: 16): one
// fibre per lane would leave most of the wavefront idle, so the lanes form 64 / (r/p) groups and
// every group takes its own far pair of the row (pairs e0 + g, e0 + g + groups, ...), with its
// own LDS buffer and its own accumulators.  The factor matrices then differ between the groups,
// so the table of the depth is staged in LDS once per target.  At the end the accumulators of the
// groups are added in a fixed order.
template <int PN>
__global__ __launch_bounds__(64) void m2l_kron_small_kernel(const int32_t *__restrict__ cellT,
                                                            const int32_t *__restrict__ cellS,
                                                            const uint64_t *__restrict__ far_ptr,
                                                            const uint32_t *__restrict__ far_col, int64_t nb, int D,
                                                            int r, const float *__restrict__ G, KronShape S,
                                                            const float *__restrict__ W, float *__restrict__ V) {
    extern __shared__ float lds[];   // [groups][r] buffers, then the table [D][no][PN][PN]
    const int64_t a = block_index();
    if (a >= nb) return;
    const uint64_t e0 = far_ptr[a], e1 = far_ptr[a + 1];
    if (e0 == e1) return;
    const int lane = threadIdx.x;
    const int nfib = r / PN;
    const int ngrp = 64 / nfib;
    const int g = lane / nfib, f = lane - g * nfib;
    const bool act = g < ngrp;
    float *buf = lds + (act ? g : 0) * r;
    float *tab = lds + ngrp * r;
    const int tab_n = D * S.no * PN * PN;
    for (int i = lane; i < tab_n; i += 64) tab[i] = G[i];
    float acc[PN];
#pragma unroll
    for (int i = 0; i < PN; ++i) acc[i] = 0.f;
    int ca[F3M_MAX_DIM];
    for (int d = 0; d < D; ++d) ca[d] = cellT[a * D + d];
    auto factor = [&](int d, int cs) {
        int k = cs - ca[d] - S.omin[d];
        k = k < 0 ? 0 : (k >= S.no ? S.no - 1 : k);
        return tab + (d * S.no + k) * (PN * PN);
    };
    auto apply = [&](const float *gm, const float (&in)[PN], float (&out)[PN]) {
#pragma unroll
        for (int i = 0; i < PN; ++i) {
            float t = 0.f;
#pragma unroll
            for (int j = 0; j < PN; ++j) t = fmaf(gm[i * PN + j], in[j], t);
            out[i] = t;
        }
    };
    for (uint64_t e = e0; e < e1; e += (uint64_t)ngrp) {   // wave-uniform trip count
        const bool live = act && e + (uint64_t)g < e1;
        const uint32_t q = far_col[live ? e + (uint64_t)g : e];
        const float *Wq = W + (int64_t)q * r;
        __syncthreads();   // the table is in place; the last pass of the previous round has read the buffers
        if (live) {
            float in[PN], out[PN];
#pragma unroll
            for (int j = 0; j < PN; ++j) in[j] = Wq[f * PN + j];
            apply(factor(0, cellS[(int64_t)q * D]), in, out);
            if (D == 1) {
#pragma unroll
                for (int i = 0; i < PN; ++i) acc[i] += out[i];
            } else {
#pragma unroll
                for (int i = 0; i < PN; ++i) buf[f + i * nfib] = out[i];
            }
        }
        int stride = 1;   // of dimension d in the LDS layout (dimensions 1..D-1 fastest first, then 0)
        for (int d = 1; d < D; ++d) {
            __syncthreads();
            if (live) {
                const int hi = (int)(((float)f + 0.5f) * (1.f / (float)stride));   // f / stride
                const int base = hi * stride * PN + (f - hi * stride);
                float in[PN], out[PN];
#pragma unroll
                for (int j = 0; j < PN; ++j) in[j] = buf[base + j * stride];
                apply(factor(d, cellS[(int64_t)q * D + d]), in, out);
                if (d == D - 1) {
#pragma unroll
                    for (int i = 0; i < PN; ++i) acc[i] += out[i];
                } else {
#pragma unroll
                    for (int i = 0; i < PN; ++i) buf[base + i * stride] = out[i];
                }
            }
            stride *= PN;
        }
    }
    // accumulators of every group to its buffer at the flat node index i = sum_d i_d p^d, then the
    // groups are added in ascending order
    __syncthreads();
    if (act) {
        int stride = 1;
        for (int d = 2; d < D; ++d) stride *= PN;
        const int hi = (int)(((float)f + 0.5f) * (1.f / (float)stride));
#pragma unroll
        for (int i = 0; i < PN; ++i) {
            int flat;
            if (D == 1) {
                flat = i;
            } else {
                const int idx = hi * stride * PN + (f - hi * stride) + i * stride;   // LDS layout index
                const int i0 = idx / nfib;
                flat = i0 + PN * (idx - i0 * nfib);
            }
            buf[flat] = acc[i];
        }
    }
    __syncthreads();
    float *Va = V + a * r;
    for (int i = lane; i < r; i += 64) {
        float sum = 0.f;
        for (int gg = 0; gg < ngrp; ++gg) sum += lds[gg * r + i];
        Va[i] = sum;
    }
}

// Offsets (source cell - target cell) a far pair of a depth can have in dimension d.  The parents
// of a far pair are near, |O + U| < theta in every dimension (U the shift at the parents' depth),
// and a child centre lies half a child edge from its parent's: |o + u| < 2 theta + 1.  Depth 1
// has the root pair as parents, which is near whatever its distance: o in {-1, 0, 1}.  One more
// offset on either side is tabulated, and everything is cut to the cells a depth has.
static KronShape kron_shape(const f3m_plan_s &P, int level) {
    KronShape S{};
    double u[F3M_MAX_DIM];
    P.grid_shift(level, u);
    const double reach = 2.0 * (double)P.theta + 2.0, cmax = (double)((1ll << level) - 1);
    S.no = 1;
    for (int d = 0; d < P.D; ++d) {
        double lo = level == 1 ? -1.0 : std::max(-cmax, std::floor(-reach - u[d]));
        double hi = level == 1 ? 1.0 : std::min(cmax, std::ceil(reach - u[d]));
        if (hi < lo) hi = lo = std::min(std::max(lo, -cmax), cmax);   // no far pair can exist here
        S.omin[d] = (int)lo;
        S.no = std::max(S.no, (int)(hi - lo) + 1);
    }
    return S;
}

// Depths whose M2L is the grouped one (more than 32 fibres per box, far rows stored): every far row once more,
// ordered by the row-major cell index of the partner.
void build_far_orders(f3m_plan_s &P, hipStream_t st) {
    for (int l = 1; l <= P.L; ++l) {
        f3m_level &lv = P.lev[l];
        if (lv.far_sz == 0 || lv.p == 0 || lv.far_implicit || lv.r / lv.p <= 32) continue;
        lv.far_ord.alloc((size_t)lv.far_sz, &P.bytes);
        far_order_kernel<<<grid_for(lv.nb), dim3(FO_NT), 0, st>>>(lv.far_ptr.p, lv.far_col.p, P.slev(l).cell.p, P.D, l, lv.nb,
                                                                lv.far_ord.p);
        F3M_HIP(hipGetLastError());
    }
}

// per depth with far pairs: the 1-D factor matrices of the node-to-node kernel matrix, built in fp64
void upload_kron_tables(f3m_plan_s &P, hipStream_t st) {
    std::vector<std::vector<float>> host_tabs;
    for (int l = 1; l <= P.L; ++l) {
        f3m_level &lv = P.lev[l];
        if (lv.far_sz == 0 || lv.p == 0) continue;
        const int p = lv.p;
        std::vector<double> s(p);
        for (int k = 0; k < p; ++k) s[k] = p > 1 ? std::cos(M_PI * (double)k / (double)(p - 1)) : 0.0;
        const double half = 0.5 * (double)P.E / (double)(1ull << l);
        const double c = half * half / (2.0 * (double)P.gamma * (double)P.gamma);
        KronShape S = kron_shape(P, l);
        if (lv.far_implicit) {
            // the candidate-grid M2L (one point set, far ratio 2) reads one table G[o + 3][i][j], o = -3..3
            S.no = 7;
            S.omin[0] = -3;
            lv.gtab_omax = 3;
        }
        const int ndim = lv.far_implicit ? 1 : P.D;
        if (!lv.far_implicit && lv.r / p <= 32) {
            // m2l_kron_small_kernel stages the factor tables of the depth in LDS beside its far-pair buffers
            const size_t lds = (size_t)((64 / (lv.r / p)) * lv.r + P.D * S.no * p * p) * sizeof(float);
            if (lds > 64 * 1024)
                fail(F3M_ERR_UNSUPPORTED, "eta = " + std::to_string(P.theta) + " gives " + std::to_string(S.no) +
                                              " cell offsets per dimension at depth " + std::to_string(l) +
                                              ": the factor tables of the M2L exceed 64 KB of LDS for this D and interp_nodes");
        }
        double u[F3M_MAX_DIM];
        P.grid_shift(l, u);
        std::vector<float> g((size_t)ndim * S.no * p * p);
        for (int d = 0; d < ndim; ++d)
            for (int k = 0; k < S.no; ++k)
                for (int i = 0; i < p; ++i)
                    for (int j = 0; j < p; ++j) {
                        // source node minus target node in half box edges: 2 (o + u) + s_j - s_i
                        const double t = 2.0 * ((double)(S.omin[d] + k) + u[d]) + s[j] - s[i];
                        g[(((size_t)d * S.no + k) * p + i) * p + j] = (float)std::exp(-c * t * t);
                    }
        lv.gtab.alloc(g.size(), &P.bytes);
        F3M_HIP(hipMemcpyAsync(lv.gtab.p, g.data(), g.size() * sizeof(float), hipMemcpyHostToDevice, st));
        host_tabs.push_back(std::move(g));   // stays alive until the copies of all depths have been waited for
    }
    if (!host_tabs.empty()) F3M_HIP(hipStreamSynchronize(st));
}


// ------------------------------------------------------------------------------------
// partial node weights of the chunks of a box -> W, in one or two stages
static void reduce_partials(f3m_plan_s &P, f3m_level &lv, int r, float *W, hipStream_t st) {
    if (lv.nslices > 0) {
        p2m_slice_kernel<<<grid_for(lv.nslices), dim3(256), 0, st>>>(lv.slice_box.p, lv.slice_first.p, lv.chunk_first.p,
                                                                    lv.nslices, r, P.Wpart.p, P.Wslice.p);
        p2m_slice_sum_kernel<<<grid_for(lv.nb), dim3(256), 0, st>>>(lv.slice_first.p, lv.chunk_first.p, lv.nb, r,
                                                                   P.Wslice.p, W);
    } else {
        p2m_reduce_kernel<<<grid_for(lv.nb), dim3(256), 0, st>>>(lv.chunk_first.p, lv.nb, r, P.Wpart.p, W);
    }
}

// every box of the depth is exactly one chunk of the P2M / L2P work split (chunk index = box rank)
static int single_chunks(const f3m_level &lv) { return lv.max_box <= P2M_CHUNK && lv.nchunks == lv.nb ? 1 : 0; }

// g = log2(e) l^2 / (2 gamma^2) of a depth: c l^2 bounds the magnitude of the expanded exponent terms in
// box-local coordinates (|x'|^2 + |y'|^2 <= 7.5 D/3 l^2)
static double gram_exponent_scale(const f3m_plan_s &P, int l) {
    const CentreArg CL = make_centre(P, l);
    const double c = 1.4426950408889634 / (2.0 * (double)P.gamma * (double)P.gamma);
    return c * CL.edge * CL.edge;
}

// the near field of a depth runs on the Gram kernels (expanded square on the matrix cores) while g D <= 6;
// above the limit, and for the root pair of two point sets (near whatever its distance: no bound on the
// coordinates), the difference form is used
static bool gram_near_field(const f3m_plan_s &P, int l) {
    const double gl = gram_exponent_scale(P, l);
    return gl * (double)P.D <= 6.0 && gl > 1e-30 && !P.force_all_near && P.T <= 1024 && !(P.src && l == 0);
}

// Slices that a target tile of the 3-D Gram near field over the near list of depth l is cut into (1: none):
// with few target tiles and long rows several wavefronts share a tile, each on a slice of the sources.
// Tiles of the last depth may be worked in pairs by p2p_gram3_pair_kernel: one point set in 3-D on the Gram
// path.  Coordinates relative to the midpoint of a pair are up to 1.6 times those relative to a box centre in
// the products of the expanded square, so the limit on g D is that of the Gram path divided by 1.6.
bool p2p_pairs_allowed(const f3m_plan_s &P) {
    return P.D == 3 && !P.src && gram_near_field(P, P.L) && gram_exponent_scale(P, P.L) * 3.0 <= 3.75 &&
           p2p_nsplit(P, P.L, P.ntiles) == 1;
}

int p2p_nsplit(const f3m_plan_s &P, int l, int64_t ntiles) {
    const f3m_level &lv = P.lev[l];
    if (!(P.D == 3 && gram_near_field(P, l) && ntiles > 0 && ntiles < 8192 && lv.nb > 0 && P.slev(l).nb > 0)) return 1;
    const double row_sources = (double)lv.near_sz / (double)lv.nb * ((double)P.ns() / (double)P.slev(l).nb);   // per tile
    const int nsplit = (int)std::min<double>(std::min<double>(64.0, (double)cdiv(262144, ntiles)), row_sources / 2048.0);
    return nsplit < 2 ? 1 : nsplit;
}

// box_order: b and y are in the plan's box order (one-set plans), so both permutations are plain passes.
// bs_in / yn_in (both or neither): the right-hand side already gathered into box order (padded like
// the plan's own buffer) and the near-field result already computed for it; used by the products with
// several right-hand sides, whose near field is evaluated for a group of columns at once.
template <int D>
static void run_kmvm_d(f3m_plan_s &P, const float *b, float *y, hipStream_t st, bool box_order,
                       const float *bs_in = nullptr, const float *yn_in = nullptr) {
    const float *bs = bs_in ? bs_in : P.bs.p;
    const float *yn = yn_in ? yn_in : P.yn.p;
    const int64_t n = P.n;
    const float nc2 = (float)(-1.4426950408889634 / (2.0 * (double)P.gamma * (double)P.gamma));
    const int nev = 4 + 3 * (P.L + 1);
    if (!P.ev[8]) {
        // events of the kmvm stages live in ev[8..15] plus a per-depth set created lazily
        for (int k = 8; k < 12; ++k) F3M_HIP(hipEventCreate(&P.ev[k]));
    }
    (void)nev;
    const unsigned gn = (unsigned)cdiv(n, 256);
    f3m_level &leaf = P.lev[P.L];
    const float *Ys = P.Ys();   // sources in box order (the targets themselves for one point set)

    F3M_HIP(hipEventRecord(P.ev[8], st));
    if (bs_in) {
        // gathered by the caller
    } else if (box_order)
        copy_kernel<<<dim3((unsigned)cdiv(P.ns(), 256)), dim3(256), 0, st>>>(b, P.ns(), P.bs.p);
    else
        if (P.sroute())
            route_gather(*P.sroute(), b, P.bs.p, P.route_a.p, P.route_b.p, st);
        else
            gather_kernel<<<dim3((unsigned)cdiv(P.ns(), 256)), dim3(256), 0, st>>>(b, P.sperm(), P.ns(), P.bs.p);
    F3M_HIP(hipEventRecord(P.ev[9], st));
    // The near field goes to the plan's second stream (vector ALU work) and overlaps the
    // far field (matrix-core work) on the caller's stream; with no_overlap it runs in line.
    hipStream_t sn = P.side ? P.side : st;
    if (P.side) {
        F3M_HIP(hipEventRecord(P.ev_fork, st));
        F3M_HIP(hipStreamWaitEvent(P.side, P.ev_fork, 0));
    }
    F3M_HIP(hipEventRecord(P.ev_p2p0, sn));
    // exact sums over a CSR list of box pairs of one depth (target tiles given), into yn
    auto direct_pairs = [&](int l, const uint64_t *row_ptr, const uint32_t *cols, const uint32_t *tile_box,
                            const uint32_t *tile_first, int64_t ntiles, int accumulate,
                            const uint8_t *paired = nullptr) {
        f3m_level &lv = P.lev[l];
        const uint32_t *sstart = P.slev(l).start.p;
        const CentreArg CL = make_centre(P, l);
        const double gl = gram_exponent_scale(P, l);
        const bool gram = gram_near_field(P, l);
        // few target tiles with long rows: several wavefronts per tile, each on a slice of the sources
        const int nsplit = cols == lv.near_col.p ? p2p_nsplit(P, l, ntiles) : 1;
        if (nsplit > 1) {
            // the partial sums were sized when the plan was built: nothing is allocated here
            if (P.p2p_part.count < (size_t)nsplit * (size_t)n)
                fail(F3M_ERR_HIP, "internal: the plan holds no room for the split near field");
            p2p_gram3_kernel<true, 1><<<grid_for(cdiv(ntiles * nsplit, 4)), dim3(256), 0, sn>>>(
                P.Xs.p, lv.start.p, Ys, bs, sstart, lv.cell.p, row_ptr, cols, tile_box, tile_first, ntiles, (float)gl,
                (float)(1.0 / CL.edge), CL, P.yn.p, accumulate, nsplit, n, P.p2p_part.p, MultiArg{}, nullptr);
            p2p_split_sum_kernel<<<dim3(gn), dim3(256), 0, sn>>>(P.p2p_part.p, nsplit, n, P.yn.p, accumulate);
        } else if (gram && D == 3) {
            if (ntiles > 0)
                p2p_gram3_kernel<false, 1><<<grid_for(cdiv(ntiles, 4)), dim3(256), 0, sn>>>(
                    P.Xs.p, lv.start.p, Ys, bs, sstart, lv.cell.p, row_ptr, cols, tile_box, tile_first, ntiles,
                    (float)gl, (float)(1.0 / CL.edge), CL, P.yn.p, accumulate, 1, n, nullptr, MultiArg{}, paired);
        }
        else if (gram)
            p2p_mfma_kernel<D><<<grid_for(cdiv(ntiles, 4)), dim3(256), 0, sn>>>(
                P.Xs.p, lv.start.p, Ys, bs, sstart, lv.cell.p, row_ptr, cols, tile_box, tile_first, ntiles, (float)gl,
                (float)(1.0 / CL.edge), CL, P.yn.p, accumulate);
        else
            p2p_kernel<D><<<grid_for(ntiles), dim3(64), 0, sn>>>(P.Xs.p, lv.start.p, Ys, bs, sstart, row_ptr, cols,
                                                                tile_box, tile_first, ntiles, nc2, P.yn.p, accumulate);
        F3M_HIP(hipGetLastError());
    };
    if (yn_in) {
        // computed by the caller
    } else if (leaf.near_sz == 0) {
        // every pair was interpolated (smooth field, Sec. 4.3) or summed at its own depth (small field)
        zero_kernel<<<dim3(gn), dim3(256), 0, sn>>>(P.yn.p, n);
    } else {
        if (P.npairs > 0) {
            // the first runs of paired boxes two at a time, every other big tile on its own
            const CentreArg CL = make_centre(P, P.L);
            p2p_gram3_pair_kernel<<<grid_for(cdiv(P.npairs, 4)), dim3(256), 0, sn>>>(
                P.Xs.p, leaf.start.p, bs, leaf.cell.p, leaf.near_ptr.p, leaf.near_col.p, P.pair_box.p, P.npairs, P.T,
                (float)gram_exponent_scale(P, P.L), (float)(1.0 / CL.edge), CL, P.yn.p);
            F3M_HIP(hipGetLastError());
            direct_pairs(P.L, leaf.near_ptr.p, leaf.near_col.p, P.rtile_box.p, P.rtile_first.p, P.nrtiles, 0,
                         P.paired.p);
        } else {
            direct_pairs(P.L, leaf.near_ptr.p, leaf.near_col.p, P.tile_box.p, P.tile_first.p, P.ntiles, 0);
        }
        // last runs with few targets: sources on the lanes
        if (P.notiles > 0)
            p2p_small_kernel<D, overflow_targets(D)><<<grid_for(cdiv(P.notiles, 4)), dim3(256), 0, sn>>>(
                P.Xs.p, leaf.start.p, Ys, bs, P.slev(P.L).start.p, leaf.near_ptr.p, leaf.near_col.p, P.otile_box.p,
                P.otile_first.p, P.notiles, nc2, P.yn.p, 1, 0);
    }
    // small-field pairs of every depth (Sec. 4.2), added on top
    for (int l = 1; l <= P.L && !yn_in; ++l) {
        f3m_level &lv = P.lev[l];
        if (lv.small_sz > 0) {
            p2p_small_kernel<D, small_tt<D>()><<<grid_for(cdiv(lv.sm_ntiles, 4)), dim3(256), 0, sn>>>(
                P.Xs.p, lv.start.p, Ys, bs, P.slev(l).start.p, lv.small_ptr.p, lv.small_col.p, lv.sm_tile_box.p,
                lv.sm_tile_first.p, lv.sm_ntiles, nc2, P.yn.p, 0, 1);
            F3M_HIP(hipGetLastError());
        }
    }
    F3M_HIP(hipGetLastError());
    F3M_HIP(hipEventRecord(P.ev_p2p1, sn));
    if (P.side) F3M_HIP(hipEventRecord(P.ev_join, P.side));
    zero_kernel<<<dim3(gn), dim3(256), 0, st>>>(P.ys.p, n);
    F3M_HIP(hipEventRecord(P.ev[10], st));
    // six events per depth: [0,1] bracket the upward pass (P2M or M2M), [2,3] the M2L, [4,5] the
    // downward pass (L2L and/or L2P) of that depth
    P.far_events.resize((size_t)(P.L + 1) * 6, nullptr);
    auto level_events = [&](int l) {
        hipEvent_t *ev = &P.far_events[(size_t)l * 6];
        for (int k = 0; k < 6; ++k)
            if (!ev[k]) F3M_HIP(hipEventCreate(&ev[k]));
        return ev;
    };
    const bool tree = P.tree_lmin > 0;   // D = 3, 4 nodes per dimension on depths tree_lmin..tree_lmax
    // node weights of the source boxes of a depth, from the points, into P.W (the boxes its chunk list names)
    auto p2m_depth = [&](int l) {
        f3m_level &lv = P.lev[l];
        f3m_level &sv = P.slev(l);
        const int p = lv.p, r = lv.r;
        const NodeArg N = make_nodes(p);
        const CentreArg CS = make_centre(P, l, true);   // source grid
        size_t sh = (size_t)(FF_TP * D * p + FF_TP) * sizeof(float);
        if (D == 3 && p == 4 && single_chunks(sv))
            p2m34_pair_kernel<<<grid_for(cdiv(sv.nb, 2 * P2M_NPAIR)), dim3(64), 0, st>>>(Ys, bs, sv.start.p, sv.cell.p, sv.nb,
                                                                                        CS, P.W.p);
        else if (D == 3 && p == 4)
            p2m34_kernel<<<grid_for(cdiv(sv.nchunks, P2M_NCH)), dim3(64), 0, st>>>(Ys, bs, sv.start.p, sv.cell.p,
                                                                  sv.chunk_box.p, sv.chunk_first.p, sv.nchunks, CS,
                                                                  P.W.p, P.Wpart.p, single_chunks(sv));
        else if (r <= 64)
            p2m_kernel<D, 64><<<grid_for(sv.nchunks), dim3(64), sh, st>>>(
                Ys, bs, sv.start.p, sv.cell.p, sv.chunk_box.p, sv.chunk_first.p, sv.nchunks, p, r, CS, N,
                P.W.p, P.Wpart.p);
        else
            p2m_kernel<D, 256><<<grid_for(sv.nchunks), dim3(256), sh, st>>>(
                Ys, bs, sv.start.p, sv.cell.p, sv.chunk_box.p, sv.chunk_first.p, sv.nchunks, p, r, CS, N,
                P.W.p, P.Wpart.p);
        F3M_HIP(hipGetLastError());
        if (sv.max_box > P2M_CHUNK)   // some box has several chunks
            reduce_partials(P, sv, r, P.W.p, st);
        F3M_HIP(hipGetLastError());
    };
    // M2L of a depth from its far list, factor by factor; rows of V whose far row is empty are left alone
    auto kron_m2l = [&](int l, const float *W, float *V) {
        f3m_level &lv = P.lev[l];
        f3m_level &sv = P.slev(l);
        const int p = lv.p, r = lv.r;
        const KronShape KS = kron_shape(P, l);
        const int nfib = r / p;
        if (nfib <= 32) {   // several far pairs per wavefront
            const size_t sh = (size_t)((64 / nfib) * r + D * KS.no * p * p) * sizeof(float);
            auto launch = [&](auto kern) {
                kern<<<grid_for(lv.nb), dim3(64), sh, st>>>(lv.cell.p, sv.cell.p, lv.far_ptr.p, lv.far_col.p, lv.nb, D, r,
                                                            lv.gtab.p, KS, W, V);
            };
            switch (p) {
                case 2: launch(m2l_kron_small_kernel<2>); break;
                case 3: launch(m2l_kron_small_kernel<3>); break;
                case 4: launch(m2l_kron_small_kernel<4>); break;
                case 5: launch(m2l_kron_small_kernel<5>); break;
                case 6: launch(m2l_kron_small_kernel<6>); break;
                case 7: launch(m2l_kron_small_kernel<7>); break;
                case 8: launch(m2l_kron_small_kernel<8>); break;
                default: fail(F3M_ERR_UNSUPPORTED, "interp_nodes must be in [2,8]");
            }
        } else {
            if (!lv.far_ord.p) fail(F3M_ERR_HIP, "internal: the far rows of this depth have not been ordered");
            auto launch = [&](auto kern) {
                kern<<<grid_for(lv.nb), dim3(256), 0, st>>>(lv.cell.p, sv.cell.p, lv.far_ptr.p, lv.far_ord.p, lv.nb, lv.gtab.p,
                                                           KS, W, V);
            };
            // every (nodes per dimension, D) with more than 32 fibres and at most 4096 nodes
            switch (p * 8 + D) {
                case 2 * 8 + 7: launch(m2l_kron_grouped_kernel<2, 7>); break;
                case 3 * 8 + 5: launch(m2l_kron_grouped_kernel<3, 5>); break;
                case 3 * 8 + 6: launch(m2l_kron_grouped_kernel<3, 6>); break;
                case 3 * 8 + 7: launch(m2l_kron_grouped_kernel<3, 7>); break;
                case 4 * 8 + 4: launch(m2l_kron_grouped_kernel<4, 4>); break;
                case 4 * 8 + 5: launch(m2l_kron_grouped_kernel<4, 5>); break;
                case 4 * 8 + 6: launch(m2l_kron_grouped_kernel<4, 6>); break;
                case 5 * 8 + 4: launch(m2l_kron_grouped_kernel<5, 4>); break;
                case 5 * 8 + 5: launch(m2l_kron_grouped_kernel<5, 5>); break;
                case 6 * 8 + 3: launch(m2l_kron_grouped_kernel<6, 3>); break;
                case 6 * 8 + 4: launch(m2l_kron_grouped_kernel<6, 4>); break;
                case 7 * 8 + 3: launch(m2l_kron_grouped_kernel<7, 3>); break;
                case 7 * 8 + 4: launch(m2l_kron_grouped_kernel<7, 4>); break;
                case 8 * 8 + 3: launch(m2l_kron_grouped_kernel<8, 3>); break;
                case 8 * 8 + 4: launch(m2l_kron_grouped_kernel<8, 4>); break;
                default: fail(F3M_ERR_UNSUPPORTED, "no M2L kernel for this number of nodes and dimensions");
            }
        }
        F3M_HIP(hipGetLastError());
    };
    // ---- depths that are handled on their own, straight from the points (Fig. 4 steps 1-3)
    for (int l = 1; l <= P.L; ++l) {
        f3m_level &lv = P.lev[l];
        // no far pairs, dropped by the adaptive rule (Sec. 4.3), or part of the band below
        if (lv.far_sz == 0 || lv.p == 0 || (tree && l >= P.tree_lmin && l <= P.tree_lmax)) continue;
        const int p = lv.p, r = lv.r;
        const NodeArg N = make_nodes(p);
        hipEvent_t *ev = level_events(l);
        const CentreArg C = make_centre(P, l);          // target grid
        F3M_HIP(hipEventRecord(ev[0], st));
        p2m_depth(l);
        F3M_HIP(hipEventRecord(ev[1], st));
        F3M_HIP(hipEventRecord(ev[2], st));
        if (!(lv.far_implicit && run_m2l_stencil(P, l, P.W.p, P.V.p, st))) kron_m2l(l, P.W.p, P.V.p);
        F3M_HIP(hipEventRecord(ev[3], st));
        F3M_HIP(hipEventRecord(ev[4], st));
        {
            size_t sh = (size_t)(r + P2M_CHUNK * (D * p + 1)) * sizeof(float);
            if (D == 3 && p == 4)
                l2p34_kernel<<<grid_for(cdiv(lv.nchunks, L2P_NCH)), dim3(64), 0, st>>>(P.Xs.p, lv.start.p, lv.cell.p, lv.far_ptr.p,
                                                                      lv.chunk_box.p, lv.chunk_first.p, lv.nchunks, C,
                                                                      P.V.p, P.ys.p, single_chunks(lv));
            else
                l2p_kernel<D><<<grid_for(lv.nchunks), dim3(P2M_CHUNK), sh, st>>>(
                    P.Xs.p, lv.start.p, lv.cell.p, lv.far_ptr.p, lv.chunk_box.p, lv.chunk_first.p, lv.nchunks, p, r, C, N,
                    P.V.p, P.ys.p);
            F3M_HIP(hipGetLastError());
        }
        F3M_HIP(hipEventRecord(ev[5], st));
    }
    // ---- depths tree_lmin..tree_lmax: P2M at the last depth of the band, weights passed upward,
    //      M2L per depth, potentials passed downward, one L2P at the last depth of the band
    if (tree) {
        // One point set: node weights from the points at the last depth of the band and upward from
        // there.  Two point sets: only the targets' side uses the tree; the node weights of a depth come
        // from the points of the source boxes that its far rows name (the sources' tree may hold many
        // more boxes than are ever used, and a pass over all of them costs more than it saves).
        const int L = P.tree_lmax;
        const int r = 64;
        f3m_level &lf = P.lev[L];
        if (!P.src) {
            {
                hipEvent_t *ev = level_events(L);
                F3M_HIP(hipEventRecord(ev[0], st));
                if (single_chunks(lf))
                    p2m34_pair_kernel<<<grid_for(cdiv(lf.nb, 2 * P2M_NPAIR)), dim3(64), 0, st>>>(P.Xs.p, bs, lf.start.p, lf.cell.p,
                                                                                                lf.nb, make_centre(P, L), lf.Wl.p);
                else
                    p2m34_kernel<<<grid_for(cdiv(lf.nchunks, P2M_NCH)), dim3(64), 0, st>>>(P.Xs.p, bs, lf.start.p, lf.cell.p, lf.chunk_box.p,
                                                                          lf.chunk_first.p, lf.nchunks, make_centre(P, L),
                                                                          lf.Wl.p, P.Wpart.p, single_chunks(lf));
                F3M_HIP(hipGetLastError());
                if (lf.max_box > P2M_CHUNK)   // some box has several chunks
                    reduce_partials(P, lf, r, lf.Wl.p, st);
                F3M_HIP(hipGetLastError());
                F3M_HIP(hipEventRecord(ev[1], st));
            }
            for (int l = L - 1; l >= P.tree_lmin; --l) {
                f3m_level &lv = P.lev[l], &dn = P.lev[l + 1];
                hipEvent_t *ev = level_events(l);
                F3M_HIP(hipEventRecord(ev[0], st));
                m2m34_kernel<<<grid_for(lv.nb), dim3(64), 0, st>>>(lv.cstart.p, dn.key.p, lv.nb, P.transfer.p, dn.Wl.p, lv.Wl.p);
                F3M_HIP(hipGetLastError());
                F3M_HIP(hipEventRecord(ev[1], st));
            }
        }
        for (int l = P.tree_lmin; l <= L; ++l) {
            f3m_level &lv = P.lev[l];
            hipEvent_t *ev = level_events(l);
            if (P.src) {
                F3M_HIP(hipEventRecord(ev[0], st));
                p2m_depth(l);
                F3M_HIP(hipEventRecord(ev[1], st));
            }
            F3M_HIP(hipEventRecord(ev[2], st));
            if (lv.far_implicit) {
                if (!run_m2l_stencil(P, l, lv.Wl.p, lv.Vl.p, st, true))   // Wl ends with a row of zeros
                    fail(F3M_ERR_HIP, "internal: depth outside the candidate-grid M2L");
            } else {
                // from the far list: the potentials of the boxes without far partners must read zero
                zero_kernel<<<dim3((unsigned)cdiv(lv.nb * (int64_t)r, 256)), dim3(256), 0, st>>>(lv.Vl.p, lv.nb * (int64_t)r);
                kron_m2l(l, P.src ? P.W.p : lv.Wl.p, lv.Vl.p);
            }
            F3M_HIP(hipEventRecord(ev[3], st));
        }
        for (int l = P.tree_lmin + 1; l <= L; ++l) {
            f3m_level &lv = P.lev[l], &up = P.lev[l - 1];
            hipEvent_t *ev = level_events(l);
            F3M_HIP(hipEventRecord(ev[4], st));
            l2l34_kernel<<<grid_for(up.nb), dim3(64), 0, st>>>(up.cstart.p, lv.key.p, up.nb, P.transfer.p, up.Vl.p, lv.Vl.p);
            F3M_HIP(hipGetLastError());
            if (l < L) F3M_HIP(hipEventRecord(ev[5], st));
        }
        {
            hipEvent_t *ev = level_events(L);
            if (P.tree_lmin == L) F3M_HIP(hipEventRecord(ev[4], st));
            l2p34_kernel<<<grid_for(cdiv(lf.nchunks, L2P_NCH)), dim3(64), 0, st>>>(P.Xs.p, lf.start.p, lf.cell.p, nullptr, lf.chunk_box.p,
                                                                  lf.chunk_first.p, lf.nchunks, make_centre(P, L),
                                                                  lf.Vl.p, P.ys.p, single_chunks(lf));
            F3M_HIP(hipGetLastError());
            F3M_HIP(hipEventRecord(ev[5], st));
        }
        // the lowest tree depth has no downward pass of its own
        {
            hipEvent_t *ev = level_events(P.tree_lmin);
            if (P.tree_lmin < L) {
                F3M_HIP(hipEventRecord(ev[4], st));
                F3M_HIP(hipEventRecord(ev[5], st));
            }
        }
    }
    if (P.side) F3M_HIP(hipStreamWaitEvent(st, P.ev_join, 0));
    F3M_HIP(hipEventRecord(P.ev[11], st));
    if (box_order) {
        add_kernel<<<dim3(gn), dim3(256), 0, st>>>(P.ys.p, yn, n, y);
        F3M_HIP(hipGetLastError());
    } else if (P.route) {
        route_scatter(*P.route, P.ys.p, yn, y, P.route_a.p, P.route_b.p, st);
    } else {
        scatter_kernel<<<dim3(gn), dim3(256), 0, st>>>(P.ys.p, yn, P.perm.p, n, y);
        F3M_HIP(hipGetLastError());
    }
    if (!P.ev[12]) F3M_HIP(hipEventCreate(&P.ev[12]));
    F3M_HIP(hipEventRecord(P.ev[12], st));
    // A product that is being captured into a graph has no times: its event records are nodes of the graph, not
    // time stamps the host can read (f3m_stage_times then reports the stages of the plan only).
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    F3M_HIP(hipStreamIsCapturing(st, &capturing));
    P.have_kmvm_times = capturing == hipStreamCaptureStatusNone;
}

// Products with several right-hand sides: column j of B (ns entries from B + j ldb) gives column j of Y
// (n entries at Y + j ldy).  Where the near field runs on the D = 3 Gram kernel, it is evaluated for groups
// of up to 4 columns at once (the exponentials, the dominant cost, are shared); everything else is done
// column by column with the kernels of the single product.  Otherwise: m single products.
void run_kmvm_multi(f3m_plan_s &P, const float *B, int64_t ldb, float *Y, int64_t ldy, int m, hipStream_t st) {
    const int64_t n = P.n, ns = P.ns();
    f3m_level &leaf = P.lev[P.L];
    const CentreArg CL = make_centre(P, P.L);
    const double gl = 1.4426950408889634 / (2.0 * (double)P.gamma * (double)P.gamma) * CL.edge * CL.edge;
    // the conditions under which the single product uses the plain D = 3 Gram kernel for its near field
    const bool fused = m > 1 && P.D == 3 && gl * 3.0 <= 6.0 && gl > 1e-30 && !P.force_all_near && P.T <= 1024 &&
                       !(P.src && P.L == 0) && P.rho == 0 && leaf.near_sz > 0 && P.ntiles >= 8192;
    if (!fused) {
        for (int j = 0; j < m; ++j) run_kmvm(P, B + (int64_t)j * ldb, Y + (int64_t)j * ldy, st);
        return;
    }
    const size_t bs_stride = (size_t)ns + PAD_POINTS;
    if (!P.multi_bs.p) {
        P.multi_bs.alloc(4 * bs_stride, &P.bytes);
        P.multi_yn.alloc(4 * (size_t)n, &P.bytes);
        F3M_HIP(hipMemsetAsync(P.multi_bs.p, 0, 4 * bs_stride * sizeof(float), st));   // the padding stays zero
    }
    for (int j0 = 0; j0 < m; j0 += 4) {
        const int mb = std::min(4, m - j0);
        if (mb == 1) {
            run_kmvm(P, B + (int64_t)j0 * ldb, Y + (int64_t)j0 * ldy, st);
            break;
        }
        MultiArg MA{};
        for (int j = 0; j < mb; ++j) {
            float *bsj = P.multi_bs.p + (size_t)j * bs_stride;
            if (P.sroute())
                route_gather(*P.sroute(), B + (int64_t)(j0 + j) * ldb, bsj, P.route_a.p, P.route_b.p, st);
            else
                gather_kernel<<<dim3((unsigned)cdiv(ns, 256)), dim3(256), 0, st>>>(B + (int64_t)(j0 + j) * ldb, P.sperm(), ns, bsj);
            MA.bs[j] = bsj;
            MA.ys[j] = P.multi_yn.p + (size_t)j * (size_t)n;
        }
        F3M_HIP(hipGetLastError());
        auto launch = [&](auto kern) {
            kern<<<grid_for(cdiv(P.ntiles, 4)), dim3(256), 0, st>>>(
                P.Xs.p, leaf.start.p, P.Ys(), nullptr, P.slev(P.L).start.p, leaf.cell.p, leaf.near_ptr.p, leaf.near_col.p,
                P.tile_box.p, P.tile_first.p, P.ntiles, (float)gl, (float)(1.0 / CL.edge), CL, nullptr, 0, 1, n, nullptr, MA,
                nullptr);
        };
        if (mb == 2) launch(p2p_gram3_kernel<false, 2>);
        else if (mb == 3) launch(p2p_gram3_kernel<false, 3>);
        else launch(p2p_gram3_kernel<false, 4>);
        F3M_HIP(hipGetLastError());
        if (P.notiles > 0) {
            const float nc2 = (float)(-1.4426950408889634 / (2.0 * (double)P.gamma * (double)P.gamma));
            for (int j = 0; j < mb; ++j)
                p2p_small_kernel<3, overflow_targets(3)><<<grid_for(cdiv(P.notiles, 4)), dim3(256), 0, st>>>(
                    P.Xs.p, leaf.start.p, P.Ys(), MA.bs[j], P.slev(P.L).start.p, leaf.near_ptr.p, leaf.near_col.p,
                    P.otile_box.p, P.otile_first.p, P.notiles, nc2, MA.ys[j], 1, 0);
            F3M_HIP(hipGetLastError());
        }
        for (int j = 0; j < mb; ++j)
            run_kmvm_d<3>(P, nullptr, Y + (int64_t)(j0 + j) * ldy, st, false, MA.bs[j], MA.ys[j]);
    }
}

void run_zero(float *y, int64_t n, hipStream_t st) {
    zero_kernel<<<dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st>>>(y, n);
    F3M_HIP(hipGetLastError());
}

void run_kmvm(f3m_plan_s &P, const float *b, float *y, hipStream_t st, bool box_order) {
    switch (P.D) {
        case 1: run_kmvm_d<1>(P, b, y, st, box_order); break;
        case 2: run_kmvm_d<2>(P, b, y, st, box_order); break;
        case 3: run_kmvm_d<3>(P, b, y, st, box_order); break;
        case 4: run_kmvm_d<4>(P, b, y, st, box_order); break;
        case 5: run_kmvm_d<5>(P, b, y, st, box_order); break;
        case 6: run_kmvm_d<6>(P, b, y, st, box_order); break;
        case 7: run_kmvm_d<7>(P, b, y, st, box_order); break;
        default: fail(F3M_ERR_INVALID_ARG, "D must be in [1,7]");
    }
}

template <int D>
static void run_direct_d(const float *X, int64_t nx, const float *Y, int64_t ny, float gamma, const float *b, float *y,
                         hipStream_t st) {
    const float nc2 = (float)(-1.4426950408889634 / (2.0 * (double)gamma * (double)gamma));
    direct_kernel<D><<<dim3((unsigned)cdiv(nx, 64)), dim3(64), 0, st>>>(X, nx, Y, b, ny, nc2, y);
    F3M_HIP(hipGetLastError());
}

void run_direct(const float *X, int64_t nx, const float *Y, int64_t ny, int D, float gamma, const float *b, float *y,
                hipStream_t st) {
    switch (D) {
        case 1: run_direct_d<1>(X, nx, Y, ny, gamma, b, y, st); break;
        case 2: run_direct_d<2>(X, nx, Y, ny, gamma, b, y, st); break;
        case 3: run_direct_d<3>(X, nx, Y, ny, gamma, b, y, st); break;
        case 4: run_direct_d<4>(X, nx, Y, ny, gamma, b, y, st); break;
        case 5: run_direct_d<5>(X, nx, Y, ny, gamma, b, y, st); break;
        case 6: run_direct_d<6>(X, nx, Y, ny, gamma, b, y, st); break;
        case 7: run_direct_d<7>(X, nx, Y, ny, gamma, b, y, st); break;
        default: fail(F3M_ERR_INVALID_ARG, "D must be in [1,7]");
    }
}

static int rows_slices(int64_t n) { return (int)std::max<int64_t>(1, std::min<int64_t>(ROWS_MAX_SLICES, n / 4096)); }

// part: slices * m doubles of scratch, every entry of which the first kernel writes
template <int D>
static void run_rows_d(const float *X, const float *Y, int64_t n, float gamma, const float *b, const int64_t *rows,
                       int64_t m, double *y64, double *part, hipStream_t st) {
    const double nc = -1.0 / (2.0 * (double)gamma * (double)gamma);
    const int slices = rows_slices(n);
    rows_f64_kernel<D><<<dim3((unsigned)cdiv(m, 64), (unsigned)slices), dim3(64), 0, st>>>(X, Y, b, n, rows, m, nc, part);
    F3M_HIP(hipGetLastError());
    rows_f64_sum_kernel<<<dim3((unsigned)cdiv(m, 256)), dim3(256), 0, st>>>(part, m, slices, y64);
    F3M_HIP(hipGetLastError());
}

static void run_rows(const float *X, const float *Y, int64_t ny, int D, float gamma, const float *b,
                     const int64_t *rows, int64_t m, double *y64, double *part, hipStream_t st) {
    switch (D) {
        case 1: run_rows_d<1>(X, Y, ny, gamma, b, rows, m, y64, part, st); break;
        case 2: run_rows_d<2>(X, Y, ny, gamma, b, rows, m, y64, part, st); break;
        case 3: run_rows_d<3>(X, Y, ny, gamma, b, rows, m, y64, part, st); break;
        case 4: run_rows_d<4>(X, Y, ny, gamma, b, rows, m, y64, part, st); break;
        case 5: run_rows_d<5>(X, Y, ny, gamma, b, rows, m, y64, part, st); break;
        case 6: run_rows_d<6>(X, Y, ny, gamma, b, rows, m, y64, part, st); break;
        case 7: run_rows_d<7>(X, Y, ny, gamma, b, rows, m, y64, part, st); break;
        default: fail(F3M_ERR_INVALID_ARG, "D must be in [1,7]");
    }
}

void run_direct_rows_f64(const float *X, const float *Y, int64_t ny, int D, float gamma, const float *b,
                         const int64_t *rows, int64_t m, double *y64, hipStream_t st) {
    DevBuf<double> part;
    part.alloc((size_t)rows_slices(ny) * (size_t)m);
    run_rows(X, Y, ny, D, gamma, b, rows, m, y64, part.p, st);
    F3M_HIP(hipStreamSynchronize(st));  // `part` is released on return
}

// The same sums with the partial results in the library's static device array instead of an
// allocation: nothing here allocates or frees, and nothing waits for the device.
void run_direct_rows_f64_static(const float *X, int64_t n, int D, float gamma, const float *b, const int64_t *rows,
                                int64_t m, double *y64, hipStream_t st) {
    if (m > ROWS_STATIC_MAX_M)
        fail(F3M_ERR_UNSUPPORTED, "direct_kmvm_rows_f64_static: m = " + std::to_string(m) + " rows exceed the limit of " +
                                      std::to_string(ROWS_STATIC_MAX_M) + " (the static scratch holds 256 slices of that many)");
    run_rows(X, X, n, D, gamma, b, rows, m, y64, rows_static_scratch(), st);
}

}  // namespace f3m
