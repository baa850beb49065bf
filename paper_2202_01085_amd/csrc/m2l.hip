// M2L, v2 = K v1 (arXiv 2202.01085, Sec. 3 "Interpolating k(x,y)", Fig. 4 step 2), for D = 3
// with 4 nodes per dimension (r = 64 nodes per box) and the paper's far rule (ratio 2).
// Everything else (other D, node counts, far ratios) takes the Kronecker-factor kernels in kmvm.hip.
#include <algorithm>
#include <cmath>

#include "plan.h"

namespace f3m {

static dim3 grid2(int64_t count) {
    const int64_t gx = 1 << 16;
    if (count <= gx) return dim3((unsigned)(count > 0 ? count : 1), 1, 1);
    return dim3((unsigned)gx, (unsigned)cdiv(count, gx), 1);
}
__device__ inline int64_t block_index2() { return (int64_t)blockIdx.y * gridDim.x + blockIdx.x; }

// (one point set only: the candidate grid assumes that targets and sources share a grid)
bool m2l_stencil_applies(const f3m_plan_s &P) {
    return P.D == 3 && P.p == 4 && P.T == 4 && !P.force_all_near && !P.src;
}

// ------------------------------------------------------------------------------------
// M2L by sum factorisation over the candidate grid (D = 3, 4 nodes per dimension, far ratio 2).
//
// The Gaussian is a product over dimensions and the nodes are a tensor grid, so the node-to-node
// matrix of a far pair with cell offset o is G_{o_z} x G_{o_y} x G_{o_x} (Kronecker product of
// 4 x 4 factors, G_o[i][j] = exp(-(l/2)^2 (2 o + s_j - s_i)^2 / (2 gamma^2))).  The candidates
// of a target are the children of the boxes near its parent: a 6 x 6 x 6 grid of cells around
// the parent, of which the 3 x 3 x 3 block around the target is near and the rest far.  Hence
//   V_t = sum_cz G_{o_z} [ sum_cy G_{o_y} [ sum_{cx far} G_{o_x} W_(cx,cy,cz) ] ]
// with the x factor applied once per far candidate (189), the y factor once per line of the
// grid (36) and the z factor once per plane (6): the same sums as 189 dense 64 x 64 products,
// reordered, in 231 x 256 instead of 189 x 4096 multiply-adds.
//
// One workgroup per parent box: its 8 wavefronts first copy the node weights of all
// candidates (<= 216 rows of 64 floats, read once per parent instead of once per target)
// into LDS at their grid position, then wavefront w handles the child with parity w: lane =
// node (ix + 4 iy + 16 iz).  The x factor needs the other three entries of the lane's quad:
// DPP quad permutations; the y and z factors use ds_bpermute.  The factor entries a lane
// needs (6 candidate coordinates x 4 rotations x 3 dimensions) sit in registers.
// ------------------------------------------------------------------------------------
constexpr int ST_CAND = 216;

__global__ __launch_bounds__(512) void m2l_stencil_kernel(const uint64_t *__restrict__ up_near_ptr,
                                                          const uint32_t *__restrict__ up_near_col,
                                                          const uint32_t *__restrict__ up_cstart,
                                                          const int32_t *__restrict__ up_cell,
                                                          const int32_t *__restrict__ cell,
                                                          const uint32_t *__restrict__ key, int64_t nparents,
                                                          int64_t per_xcd, const float *__restrict__ G, int all_far,
                                                          const uint32_t *__restrict__ start, uint32_t rho,
                                                          const float *__restrict__ W, float *__restrict__ V) {
    __shared__ float rows[ST_CAND * 64];
    __shared__ int present[ST_CAND];
    __shared__ uint32_t cand[ST_CAND];      // candidate k of near parent j at [8 j + k]: rank or ~0
    __shared__ int cpos[ST_CAND];           // its position in the 6 x 6 x 6 grid
    __shared__ uint32_t ccnt[ST_CAND];      // points of the candidate at a grid position (small-field rule)
    __shared__ uint32_t qfirst[27], qcount[27];
    __shared__ float gs[7 * 16];            // the factor table
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    // consecutive parents (neighbours in space) on the same XCD, so that its L2 serves the overlap
    const int64_t bi = block_index2();
    const int64_t pb = (bi & 7) * per_xcd + (bi >> 3);
    if ((bi >> 3) >= per_xcd || pb >= nparents) return;
    // the boxes near the parent (at most 27 with far ratio 2) and their child ranges
    if (tid < 27) {
        const uint64_t e = up_near_ptr[pb] + tid;
        uint32_t first = 0, count = 0;
        if (e < up_near_ptr[pb + 1]) {
            const uint32_t q = up_near_col[e];
            first = up_cstart[q];
            count = up_cstart[q + 1] - first;
        }
        qfirst[tid] = first;
        qcount[tid] = count;
    }
    if (tid < ST_CAND) present[tid] = 0;
    if (tid >= 256 && tid < 256 + 7 * 16) gs[tid - 256] = G[tid - 256];
    __syncthreads();
    if (tid < ST_CAND) {
        const int j = tid >> 3, k = tid & 7;
        uint32_t c = 0xFFFFFFFFu;
        if ((uint32_t)k < qcount[j]) {
            c = qfirst[j] + k;
            const int px = cell[(int64_t)c * 3] - 2 * up_cell[pb * 3] + 2,
                      py = cell[(int64_t)c * 3 + 1] - 2 * up_cell[pb * 3 + 1] + 2,
                      pz = cell[(int64_t)c * 3 + 2] - 2 * up_cell[pb * 3 + 2] + 2;
            const int pos = px + 6 * py + 36 * pz;     // in [0, 216): the near box is within one cell of the parent
            cpos[tid] = pos;
            present[pos] = 1;
            if (rho) ccnt[pos] = start[c + 1] - start[c];
        }
        cand[tid] = c;
    }
    __syncthreads();
    // node weights of the candidates into LDS: 27 rows per wavefront, all loads in flight together
    {
        float tmp[27];
#pragma unroll
        for (int i = 0; i < 27; ++i) {
            const uint32_t c = cand[w + 8 * i];
            tmp[i] = W[(int64_t)(c == 0xFFFFFFFFu ? 0u : c) * 64 + lane];
        }
#pragma unroll
        for (int i = 0; i < 27; ++i)
            if (cand[w + 8 * i] != 0xFFFFFFFFu) rows[cpos[w + 8 * i] * 64 + lane] = tmp[i];
    }
    __syncthreads();
    // the child with parity w, if it exists (no barrier below this point)
    uint32_t t = 0xFFFFFFFFu;
    for (uint32_t c = up_cstart[pb]; c < up_cstart[pb + 1]; ++c)
        if ((key[c] & 7u) == (uint32_t)w) t = c;
    if (t == 0xFFFFFFFFu) return;
    const int tx = w & 1, ty = (w >> 1) & 1, tz = w >> 2;
    const uint32_t tcnt = rho ? start[t + 1] - start[t] : 0u;
    // far and present candidates, one bit each: bit cx + 8 (cy + 6 cz), so that the six bits of a
    // line of the grid sit in one byte
    uint64_t mask[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        const int mm = lane + 64 * k, cx = mm & 7, ln = mm >> 3;
        bool ok = false;
        if (cx < 6 && ln < 36) {
            const int cy = ln % 6, cz = ln / 6;
            const int ox = cx - 2 - tx, oy = cy - 2 - ty, oz = cz - 2 - tz;
            // all_far: the smooth depth of Sec. 4.3, where adjacent pairs are interpolated too
            ok = present[cx + 6 * ln] != 0 && (all_far || ox * ox + oy * oy + oz * oz >= 4);
            // small field (Sec. 4.2): a pair with at most rho points is summed directly elsewhere
            if (ok && rho && tcnt + ccnt[cx + 6 * ln] <= rho) ok = false;
        }
        mask[k] = __ballot(ok);
    }
    const int ix = lane & 3, iy = (lane >> 2) & 3, iz = lane >> 4;
    // factor entries: candidate coordinate c (offset c - 2 - t_d), rotation k -> G_o[i][(i + k) % 4]
    float fx[6][4], fy[6][4], fz[6][4];
#pragma unroll
    for (int c = 0; c < 6; ++c)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            fx[c][k] = gs[(c + 1 - tx) * 16 + ix * 4 + ((ix + k) & 3)];
            fy[c][k] = gs[(c + 1 - ty) * 16 + iy * 4 + ((iy + k) & 3)];
            fz[c][k] = gs[(c + 1 - tz) * 16 + iz * 4 + ((iz + k) & 3)];
        }
    int ylane[4], zlane[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        ylane[k] = ix + 4 * ((iy + k) & 3) + 16 * iz;
        zlane[k] = ix + 4 * iy + 16 * ((iz + k) & 3);
    }
    float acc = 0.f;
#pragma unroll
    for (int cz = 0; cz < 6; ++cz) {
        float plane = 0.f;
#pragma unroll
        for (int cy = 0; cy < 6; ++cy) {
            float line = 0.f;
            // the six rows of the line are read unconditionally (rows of absent candidates hold
            // stale data and are skipped below), so one wait covers them
            float v[6];
#pragma unroll
            for (int cx = 0; cx < 6; ++cx) v[cx] = rows[(cx + 6 * cy + 36 * cz) * 64 + lane];
            // line += sum_k fx[cx][k] * (entry k places further in the lane's quad); the row value
            // comes straight from the LDS read, so no vector-ALU write precedes the DPP reads of it
            auto xfactor = [&](int cx) {
                asm("v_fmac_f32 %0, %2, %1\n\t"
                    "v_fmac_f32_dpp %0, %1, %3 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                    "v_fmac_f32_dpp %0, %1, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                    "v_fmac_f32_dpp %0, %1, %5 quad_perm:[3,0,1,2] row_mask:0xf bank_mask:0xf bound_ctrl:1"
                    : "+v"(line)
                    : "v"(v[cx]), "v"(fx[cx][0]), "v"(fx[cx][1]), "v"(fx[cx][2]), "v"(fx[cx][3]));
            };
            const int ln = cy + 6 * cz;
            const uint32_t bits = (uint32_t)(mask[ln >> 3] >> (8 * (ln & 7))) & 0x3Fu;
            if (bits == 0x3Fu) {   // the whole line is far and present: no tests
#pragma unroll
                for (int cx = 0; cx < 6; ++cx) xfactor(cx);
            } else {
#pragma unroll
                for (int cx = 0; cx < 6; ++cx)
                    if ((bits >> cx) & 1u) xfactor(cx);
            }
            // y factor: the lane needs the entries 4, 8, 12 lanes further on in its row of 16
            // lanes (cyclically): row rotations by 12, 8, 4 to the right
            // (`line` was last written by a vector-ALU instruction: the plain multiply-add and
            // the s_nop give the two wait states that a DPP read of it needs)
            asm("v_fmac_f32 %0, %2, %1\n\t"
                "s_nop 0\n\t"
                "v_fmac_f32_dpp %0, %1, %3 row_ror:12 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                "v_fmac_f32_dpp %0, %1, %4 row_ror:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                "v_fmac_f32_dpp %0, %1, %5 row_ror:4 row_mask:0xf bank_mask:0xf bound_ctrl:1"
                : "+v"(plane)
                : "v"(line), "v"(fy[cy][0]), "v"(fy[cy][1]), "v"(fy[cy][2]), "v"(fy[cy][3]));
        }
        acc = fmaf(fz[cz][0], plane, acc);
#pragma unroll
        for (int k = 1; k < 4; ++k) acc = fmaf(fz[cz][k], __shfl(plane, zlane[k], 64), acc);
    }
    V[(int64_t)t * 64 + lane] = acc;
}

// ------------------------------------------------------------------------------------
// The same sums with the work shared between the eight children of a parent (no small field).
// The far sum of a target is the sum over ALL candidates of the 6 x 6 x 6 grid minus the sum over
// the 3 x 3 x 3 block around the target, and the sum over all candidates factorises further: the
// x factor of a candidate depends on the target's x parity only, so the line sums
//   X_tx(cy, cz) = sum_cx G_{cx-2-tx} W_(cx,cy,cz)              2 x 36 lines, 6 applications each
// serve four targets each, the plane sums
//   Y_{tx,ty}(cz) = sum_cy G_{cy-2-ty} X_tx(cy, cz)             4 x 6 planes, 6 applications each
// serve two, and a target needs only
//   V_all = sum_cz G_{cz-2-tz} Y_{tx,ty}(cz)                    6 applications
//   V_t   = V_all - sum over the near block, again by lines and planes: 27 + 9 + 3 applications.
// Per parent 432 + 144 + 8 x (6 + 39) = 936 applications of a 4 x 4 factor to a 64-vector instead
// of 8 x 231.  Rows of absent candidates are zero in LDS, so no masks are needed.  The
// subtraction costs no accuracy that matters: |near part| / |far part| is of order one for wide
// kernels, and for narrow ones both are part of a result dominated by the near field itself.
// all_far (the smooth depth of Sec. 4.3, every candidate interpolated): no subtraction.
// ------------------------------------------------------------------------------------
// tables for it, made once per plan and depth: for every parent the rank of the candidate at each
// position of its 6 x 6 x 6 grid (~0: no such box) and its child of each parity (~0: none), so that a
// workgroup starts with one table read instead of a chain of four dependent ones (near list ->
// child ranges -> cells -> rows), which is what bounded the kernel
__global__ __launch_bounds__(256) void stencil_table_kernel(const uint64_t *__restrict__ up_near_ptr,
                                                            const uint32_t *__restrict__ up_near_col,
                                                            const uint32_t *__restrict__ up_cstart,
                                                            const int32_t *__restrict__ up_cell,
                                                            const int32_t *__restrict__ cell,
                                                            const uint32_t *__restrict__ key, int64_t nparents,
                                                            uint32_t *__restrict__ cand_tab,
                                                            uint32_t *__restrict__ child_tab) {
    const int64_t pb = block_index2();
    if (pb >= nparents) return;
    const int tid = threadIdx.x;
    if (tid < ST_CAND) {
        const int j = tid >> 3, k = tid & 7;
        const uint64_t e = up_near_ptr[pb] + j;
        if (e < up_near_ptr[pb + 1]) {
            const uint32_t q = up_near_col[e];
            const uint32_t first = up_cstart[q], count = up_cstart[q + 1] - first;
            if ((uint32_t)k < count) {
                const uint32_t c = first + k;
                const int px = cell[(int64_t)c * 3] - 2 * up_cell[pb * 3] + 2,
                          py = cell[(int64_t)c * 3 + 1] - 2 * up_cell[pb * 3 + 1] + 2,
                          pz = cell[(int64_t)c * 3 + 2] - 2 * up_cell[pb * 3 + 2] + 2;
                // in [0, 6) each: a near box is within one cell of the parent
                cand_tab[pb * ST_CAND + px + 6 * py + 36 * pz] = c;
            }
        }
    } else if (tid < ST_CAND + 8) {
        const uint32_t w = (uint32_t)(tid - ST_CAND);
        for (uint32_t c = up_cstart[pb]; c < up_cstart[pb + 1]; ++c)
            if ((key[c] & 7u) == w) child_tab[pb * 8 + w] = c;
    }
}

// ZROW: W has a row of zeros behind its last box (index zero_row): an absent candidate (~0 in the table)
// reads that row, which saves the compare-and-select pairs around every load.
template <bool ZROW>
__global__ __launch_bounds__(512) void m2l_stencil_shared_kernel(const uint32_t *__restrict__ cand_tab,
                                                                 const uint32_t *__restrict__ child_tab,
                                                                 int64_t nparents, int64_t per_xcd,
                                                                 const float *__restrict__ G, int all_far,
                                                                 uint32_t zero_row,
                                                                 const float *__restrict__ W, float *__restrict__ V) {
    __shared__ float rows[ST_CAND * 64];
    __shared__ float xl[2 * 36 * 64];       // X_tx(cy, cz) at [(tx * 36 + cy + 6 cz) * 64 + node]
    __shared__ float yp[4 * 6 * 64];        // Y_{tx,ty}(cz) at [((tx + 2 ty) * 6 + cz) * 64 + node]
    // the candidate ranks are needed only while the rows are loaded and live in the memory of xl
    // (two workgroups per compute unit fit only below 80 KB each)
    uint32_t *cand = reinterpret_cast<uint32_t *>(xl);
    __shared__ float gs[7 * 16];            // the factor table
    // (the wavefront's number in a scalar register: the row addresses are then formed by scalar instructions)
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // consecutive parents (neighbours in space) on the same XCD, so that its L2 serves the overlap
    const int64_t bi = block_index2();
    const int64_t pb = (bi & 7) * per_xcd + (bi >> 3);
    if ((bi >> 3) >= per_xcd || pb >= nparents) return;
    if (tid < ST_CAND) cand[tid] = cand_tab[pb * ST_CAND + tid];
    if (tid >= 256 && tid < 256 + 7 * 16) gs[tid - 256] = G[tid - 256];
    const uint32_t t = child_tab[pb * 8 + w];   // the child with parity w (wave-uniform), or ~0
    __syncthreads();
    // node weights of the candidates into LDS at their grid position, zeros for absent ones: 27 rows
    // per wavefront, all loads in flight together
    {
        float tmp[27];
        if constexpr (ZROW) {
#pragma unroll
            for (int i = 0; i < 27; ++i) tmp[i] = W[(int64_t)min(cand[w + 8 * i], zero_row) * 64 + lane];
#pragma unroll
            for (int i = 0; i < 27; ++i) rows[(w + 8 * i) * 64 + lane] = tmp[i];
        } else {
#pragma unroll
            for (int i = 0; i < 27; ++i) {
                const uint32_t c = cand[w + 8 * i];
                tmp[i] = W[(int64_t)(c == 0xFFFFFFFFu ? 0u : c) * 64 + lane];
            }
#pragma unroll
            for (int i = 0; i < 27; ++i) rows[(w + 8 * i) * 64 + lane] = cand[w + 8 * i] == 0xFFFFFFFFu ? 0.f : tmp[i];
        }
    }
    __syncthreads();
    const int tx = w & 1, ty = (w >> 1) & 1, tz = w >> 2;
    const int ix = lane & 3, iy = (lane >> 2) & 3, iz = lane >> 4;
    // out += sum_k f[k] * (entry k places further on in the lane's quad / row of 16 / wavefront);
    // the input always comes straight from an LDS read (no vector-ALU write precedes the DPP reads)
    auto xapply = [&](float &out, float v, const float (&f)[4]) {
        asm("v_fmac_f32 %0, %2, %1\n\t"
            "v_fmac_f32_dpp %0, %1, %3 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %0, %1, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %0, %1, %5 quad_perm:[3,0,1,2] row_mask:0xf bank_mask:0xf bound_ctrl:1"
            : "+v"(out)
            : "v"(v), "v"(f[0]), "v"(f[1]), "v"(f[2]), "v"(f[3]));
    };
    auto yapply = [&](float &out, float v, const float (&f)[4]) {
        asm("v_fmac_f32 %0, %2, %1\n\t"
            "s_nop 0\n\t"
            "v_fmac_f32_dpp %0, %1, %3 row_ror:12 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %0, %1, %4 row_ror:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %0, %1, %5 row_ror:4 row_mask:0xf bank_mask:0xf bound_ctrl:1"
            : "+v"(out)
            : "v"(v), "v"(f[0]), "v"(f[1]), "v"(f[2]), "v"(f[3]));
    };
    // the first application of a sum: out = ..., no zeroed accumulator to start from
    auto xfirst = [&](float &out, float v, const float (&f)[4]) {
        asm("v_mul_f32 %0, %2, %1\n\t"
            "v_fmac_f32_dpp %0, %1, %3 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %0, %1, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %0, %1, %5 quad_perm:[3,0,1,2] row_mask:0xf bank_mask:0xf bound_ctrl:1"
            : "=&v"(out)
            : "v"(v), "v"(f[0]), "v"(f[1]), "v"(f[2]), "v"(f[3]));
    };
    auto yfirst = [&](float &out, float v, const float (&f)[4]) {
        asm("v_mul_f32 %0, %2, %1\n\t"
            "s_nop 0\n\t"
            "v_fmac_f32_dpp %0, %1, %3 row_ror:12 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %0, %1, %4 row_ror:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
            "v_fmac_f32_dpp %0, %1, %5 row_ror:4 row_mask:0xf bank_mask:0xf bound_ctrl:1"
            : "=&v"(out)
            : "v"(v), "v"(f[0]), "v"(f[1]), "v"(f[2]), "v"(f[3]));
    };
    int zlane[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) zlane[k] = ix + 4 * iy + 16 * ((iz + k) & 3);
    auto zapply = [&](float &out, float v, const float (&f)[4]) {
        out = fmaf(f[0], v, out);
#pragma unroll
        for (int k = 1; k < 4; ++k) out = fmaf(f[k], __shfl(v, zlane[k], 64), out);
    };
    // factor entries for candidate coordinate c and target parity t: offset c - 2 - t, rotation k
    auto factor = [&](int c, int t, int i, float (&f)[4]) {
#pragma unroll
        for (int k = 0; k < 4; ++k) f[k] = gs[(c + 1 - t) * 16 + i * 4 + ((i + k) & 3)];
    };

    // ---- line sums over x: wavefront w takes x parity w & 1 and the lines (w >> 1) + 4 i, i = 0..8
    {
        float fx[6][4];
#pragma unroll
        for (int c = 0; c < 6; ++c) factor(c, tx, ix, fx[c]);
#pragma unroll
        for (int i = 0; i < 9; ++i) {
            const int ln = (w >> 1) + 4 * i;
            float v[6];
#pragma unroll
            for (int cx = 0; cx < 6; ++cx) v[cx] = rows[(cx + 6 * ln) * 64 + lane];
            float line;
            xfirst(line, v[0], fx[0]);
#pragma unroll
            for (int cx = 1; cx < 6; ++cx) xapply(line, v[cx], fx[cx]);
            xl[(tx * 36 + ln) * 64 + lane] = line;
        }
    }
    __syncthreads();
    // ---- plane sums over y: wavefront w takes the parities (w & 3) and the planes 3 (w >> 2) .. + 2
    {
        float fy[6][4];
#pragma unroll
        for (int c = 0; c < 6; ++c) factor(c, ty, iy, fy[c]);
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int cz = 3 * (w >> 2) + i;
            float v[6];
#pragma unroll
            for (int cy = 0; cy < 6; ++cy) v[cy] = xl[(tx * 36 + cy + 6 * cz) * 64 + lane];
            float plane;
            yfirst(plane, v[0], fy[0]);
#pragma unroll
            for (int cy = 1; cy < 6; ++cy) yapply(plane, v[cy], fy[cy]);
            yp[((w & 3) * 6 + cz) * 64 + lane] = plane;
        }
    }
    __syncthreads();
    // ---- the child with parity w, if it exists (no barrier below this point)
    if (t == 0xFFFFFFFFu) return;
    float acc = 0.f;
    {
        float v[6];
#pragma unroll
        for (int cz = 0; cz < 6; ++cz) v[cz] = yp[((w & 3) * 6 + cz) * 64 + lane];
#pragma unroll
        for (int cz = 0; cz < 6; ++cz) {
            float fz[4];
            factor(cz, tz, iz, fz);
            zapply(acc, v[cz], fz);
        }
    }
    if (!all_far) {
        // minus the near block: candidates t_d + 1 .. t_d + 3 in every dimension, offsets -1, 0, 1,
        // whose factors G_{-1}, G_0, G_1 sit at table entries 2, 3, 4 whatever the parity
        float nfx[3][4], nfy[3][4], nfz[3][4];
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                nfx[i][k] = gs[(i + 2) * 16 + ix * 4 + ((ix + k) & 3)];
                nfy[i][k] = gs[(i + 2) * 16 + iy * 4 + ((iy + k) & 3)];
                nfz[i][k] = gs[(i + 2) * 16 + iz * 4 + ((iz + k) & 3)];
            }
        float near = 0.f;
#pragma unroll
        for (int k3 = 0; k3 < 3; ++k3) {
            float plane = 0.f;
#pragma unroll
            for (int k2 = 0; k2 < 3; ++k2) {
                const int base = (tx + 1) + 6 * (ty + 1 + k2) + 36 * (tz + 1 + k3);
                float v[3];
#pragma unroll
                for (int k1 = 0; k1 < 3; ++k1) v[k1] = rows[(base + k1) * 64 + lane];
                float line;
                xfirst(line, v[0], nfx[0]);
#pragma unroll
                for (int k1 = 1; k1 < 3; ++k1) xapply(line, v[k1], nfx[k1]);
                yapply(plane, line, nfy[k2]);
            }
            zapply(near, plane, nfz[k3]);
        }
        acc -= near;
    }
    V[(int64_t)t * 64 + lane] = acc;
}

// candidate and child tables of a depth whose M2L runs on the candidate grid without a small field
// the tables of a depth, preset to "none"; false: the depth does not use them
bool stencil_tables_alloc(f3m_plan_s &P, int level, hipStream_t st) {
    if (!m2l_stencil_applies(P) || level < 1 || P.rho != 0) return false;
    f3m_level &lv = P.lev[level], &up = P.lev[level - 1];
    if (!lv.far_implicit || lv.far_sz == 0 || lv.p == 0) return false;
    lv.st_cand.alloc((size_t)up.nb * ST_CAND, &P.bytes);
    lv.st_child.alloc((size_t)up.nb * 8, &P.bytes);
    F3M_HIP(hipMemsetAsync(lv.st_cand.p, 0xFF, (size_t)up.nb * ST_CAND * sizeof(uint32_t), st));
    F3M_HIP(hipMemsetAsync(lv.st_child.p, 0xFF, (size_t)up.nb * 8 * sizeof(uint32_t), st));
    return true;
}

void build_stencil_tables(f3m_plan_s &P, int level, hipStream_t st) {
    if (level >= 1 && P.lev[level].st_cand.p) return;   // written by the list kernel already
    if (!stencil_tables_alloc(P, level, st)) return;
    f3m_level &lv = P.lev[level], &up = P.lev[level - 1];
    stencil_table_kernel<<<grid2(up.nb), dim3(256), 0, st>>>(up.near_ptr.p, up.near_col.p, up.cstart.p, up.cell.p,
                                                            lv.cell.p, lv.key.p, up.nb, lv.st_cand.p, lv.st_child.p);
    F3M_HIP(hipGetLastError());
}

bool run_m2l_stencil(f3m_plan_s &P, int level, const float *W, float *V, hipStream_t st, bool zero_row) {
    if (!m2l_stencil_applies(P) || level < 1) return false;
    f3m_level &lv = P.lev[level], &up = P.lev[level - 1];
    if (lv.gtab.p == nullptr || lv.gtab_omax != 3) return false;
    const int64_t per_xcd = cdiv(up.nb, 8);
    if (lv.st_cand.p) {   // no small field: the variant that shares the line and plane sums between the children
        if (zero_row)   // W carries a row of zeros at index nb
            m2l_stencil_shared_kernel<true><<<grid2(per_xcd * 8), dim3(512), 0, st>>>(
                lv.st_cand.p, lv.st_child.p, up.nb, per_xcd, lv.gtab.p, lv.smooth ? 1 : 0, (uint32_t)lv.nb, W, V);
        else
            m2l_stencil_shared_kernel<false><<<grid2(per_xcd * 8), dim3(512), 0, st>>>(
                lv.st_cand.p, lv.st_child.p, up.nb, per_xcd, lv.gtab.p, lv.smooth ? 1 : 0, 0u, W, V);
        F3M_HIP(hipGetLastError());
        return true;
    }
    m2l_stencil_kernel<<<grid2(per_xcd * 8), dim3(512), 0, st>>>(up.near_ptr.p, up.near_col.p, up.cstart.p, up.cell.p,
                                                                lv.cell.p, lv.key.p, up.nb, per_xcd, lv.gtab.p,
                                                                lv.smooth ? 1 : 0, lv.start.p, (uint32_t)P.rho, W, V);
    F3M_HIP(hipGetLastError());
    return true;
}

}  // namespace f3m
