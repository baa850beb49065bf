// Table-driven M2L, v2 = K v1 (arXiv 2202.01085, Sec. 3 "Interpolating k(x,y)", Fig. 4
// step 2), for D = 3 with 4 nodes per dimension (r = 64 nodes per box) and the paper's far
// rule (ratio 2).
//
// All boxes of a depth are congruent and the kernel depends on x - y only, so the r x r
// matrix K_pq = k(s^p_i, s^q_j) of a far pair depends on the integer cell offset o = c_q - c_p
// alone: o in [-3,3]^3, 343 matrices of 64 x 64 per depth.  For a target whose cell has
// parity c (c_d = cell_d & 1) the far partners sit at o_d in [-2-c_d, 3-c_d] minus the 27
// near offsets: 189 "slots" per parity class.  Targets of one parity class are grouped into
// tiles of 32, and for a tile and a slot the products of 32 far pairs become ONE dense
// contraction  V[64 x 32] += K_o[64 x 64] * W_gathered[64 x 32]  on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32), 64 MFMA instructions per slot, no atomics: a tile owns its
// targets.  Everything else (other D, p, far ratios) takes the general kernel in kmvm.hip.
#include <algorithm>
#include <cmath>

#include "plan.h"

namespace f3m {

typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int M2L_R = 64;
constexpr int M2L_GROUP = 4;   // tiles handled by one wavefront

struct TileBase { uint32_t b[9]; };

static dim3 grid2(int64_t count) {
    const int64_t gx = 1 << 16;
    if (count <= gx) return dim3((unsigned)(count > 0 ? count : 1), 1, 1);
    return dim3((unsigned)gx, (unsigned)cdiv(count, gx), 1);
}
__device__ inline int64_t block_index2() { return (int64_t)blockIdx.y * gridDim.x + blockIdx.x; }

static void make_slot_tables(std::vector<int32_t> &slot_of, std::vector<int32_t> &slot_oi) {
    slot_of.assign(8 * M2L_NOFF, -1);
    slot_oi.assign(8 * M2L_NSLOT, 0);
    for (int c = 0; c < 8; ++c) {
        int s = 0;
        int lo[3], hi[3];
        for (int d = 0; d < 3; ++d) {
            int cd = (c >> d) & 1;
            lo[d] = -2 - cd;
            hi[d] = 3 - cd;
        }
        for (int oz = lo[2]; oz <= hi[2]; ++oz)
            for (int oy = lo[1]; oy <= hi[1]; ++oy)
                for (int ox = lo[0]; ox <= hi[0]; ++ox) {
                    if (ox * ox + oy * oy + oz * oz < 4) continue;  // near
                    int oi = off_index(ox, oy, oz);
                    slot_of[c * M2L_NOFF + oi] = s;
                    slot_oi[c * M2L_NSLOT + s] = oi;
                    ++s;
                }
        if (s != M2L_NSLOT) fail(F3M_ERR_HIP, "internal: far slot count");
    }
}

// K_o[i][j] = exp(-|delta|^2 / (2 gamma^2)), delta_d = (l/2) (2 o_d + s_{j_d} - s_{i_d}), evaluated in
// fp64 and stored in the order the MFMA A operand is consumed:
//   ktab[oi][g][lane][e] = K_o[ mb*32 + (lane&31) ][ (lane>>5)*32 + ks ],  g*4+e = mb*32 + ks
struct NodeD { double s[4]; };
__global__ __launch_bounds__(256) void ktab_kernel(float *__restrict__ ktab, NodeD nd, double c /* (l/2)^2/(2 gamma^2) */) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)M2L_NOFF * M2L_R * M2L_R) return;
    const int oi = (int)(idx / (M2L_R * M2L_R));
    const int rem = (int)(idx % (M2L_R * M2L_R));
    const int g = rem / 256, lane = (rem % 256) / 4, e = rem % 4;
    const int q = g * 4 + e, mb = q / 32, ks = q % 32;
    const int i = mb * 32 + (lane & 31);
    const int j = (lane >> 5) * 32 + ks;
    const int o[3] = {oi % 7 - 3, (oi / 7) % 7 - 3, oi / 49 - 3};
    double r2 = 0.0;
    int ii = i, jj = j;
    for (int d = 0; d < 3; ++d) {
        double diff = 2.0 * (double)o[d] + nd.s[jj % 4] - nd.s[ii % 4];
        r2 += diff * diff;
        ii /= 4;
        jj /= 4;
    }
    ktab[idx] = (float)exp(-r2 * c);
}

struct ParityIn {
    const uint32_t *key;
    uint32_t c;
    __device__ uint64_t operator()(int64_t a) const { return (key[a] & 7u) == c; }
};
struct ParityOut {
    uint32_t *tile_box;
    uint32_t *gpos;
    uint64_t base;
    __device__ void operator()(int64_t a, uint64_t ex, uint64_t v) const {
        if (v) {
            tile_box[base + ex] = (uint32_t)a;
            gpos[a] = (uint32_t)(base + ex);
        }
    }
};

// far row of a box on a table depth, back in CSR form (ascending ranks): introspection only
__global__ __launch_bounds__(64) void far_rows_kernel(const uint32_t *__restrict__ gpos, int64_t nb,
                                                      const uint64_t *__restrict__ far_ptr,
                                                      const uint32_t *__restrict__ fpos, uint32_t *__restrict__ cols) {
    const int64_t a = block_index2() * 64 + threadIdx.x;
    if (a >= nb) return;
    const uint32_t g = gpos[a];
    const uint32_t *row = fpos + (int64_t)(g >> 5) * (M2L_NSLOT * M2L_TILE) + (g & 31);
    uint32_t *out = cols + far_ptr[a];
    const int cnt = (int)(far_ptr[a + 1] - far_ptr[a]);
    // insertion sort of the present partners into the output row
    int m = 0;
    for (int s = 0; s < M2L_NSLOT; ++s) {
        const uint32_t b = row[(int64_t)s * M2L_TILE];
        if (b == 0xFFFFFFFFu || m >= cnt) continue;
        int k = m++;
        while (k > 0 && out[k - 1] > b) { out[k] = out[k - 1]; --k; }
        out[k] = b;
    }
}

__global__ __launch_bounds__(256) void gpos_kernel(const uint32_t *__restrict__ tile_box, int64_t nlanes,
                                                   uint32_t *__restrict__ gpos) {
    const int64_t g = block_index2() * 256 + threadIdx.x;
    if (g >= nlanes) return;
    const uint32_t a = tile_box[g];
    if (a != 0xFFFFFFFFu) gpos[a] = (uint32_t)g;
}

// One wavefront per group of M2L_GROUP = 4 tiles (128 same-parity targets); no LDS, no
// barrier, so wavefronts drift apart and the matrix pipe of a SIMD always finds one of its
// two resident waves with operands ready.  Lane l: target column n = l & 31, half h = l >> 5
// of the contraction index.  Per slot the wave loads K_o once (64 values per lane, already in
// operand order: 16 contiguous 1 KB loads) and keeps it in registers for the four tiles;
// per tile B = the lane's half row of W of its far partner and 64 MFMAs go into that tile's
// two 32 x 32 accumulators (output nodes 0..31 and 32..63).
__device__ inline void m2l_tile(const float *__restrict__ W, uint32_t src, int h, const float4 (&A)[16], f16v &acc0,
                                f16v &acc1) {
    const bool has = src != 0xFFFFFFFFu;
    if (__ballot(has) == 0ull) return;
    const float4 *Bp = reinterpret_cast<const float4 *>(W + (int64_t)(has ? src : 0u) * M2L_R + h * 32);
    float4 B[8];
#pragma unroll
    for (int g = 0; g < 8; ++g) B[g] = has ? Bp[g] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int ks = 0; ks < 32; ++ks) {
        const float4 b4 = B[ks >> 2], a0 = A[ks >> 2], a1 = A[8 + (ks >> 2)];
        const int e = ks & 3;
        const float bv = e == 0 ? b4.x : e == 1 ? b4.y : e == 2 ? b4.z : b4.w;
        const float av0 = e == 0 ? a0.x : e == 1 ? a0.y : e == 2 ? a0.z : a0.w;
        const float av1 = e == 0 ? a1.x : e == 1 ? a1.y : e == 2 ? a1.z : a1.w;
        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av0, bv, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av1, bv, acc1, 0, 0, 0);
    }
}

__device__ inline void m2l_store(float *__restrict__ V, uint32_t tgt, int h, const f16v &acc0, const f16v &acc1) {
    if (tgt == 0xFFFFFFFFu) return;
    float *dst = V + (int64_t)tgt * M2L_R;
    // accumulator register v of lane (n,h) holds output node 8*(v/4) + 4*h + (v%4) of column n
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) {
        const int row = 8 * v4 + 4 * h;
        *reinterpret_cast<float4 *>(dst + row) = make_float4(acc0[4 * v4], acc0[4 * v4 + 1], acc0[4 * v4 + 2], acc0[4 * v4 + 3]);
        *reinterpret_cast<float4 *>(dst + 32 + row) = make_float4(acc1[4 * v4], acc1[4 * v4 + 1], acc1[4 * v4 + 2], acc1[4 * v4 + 3]);
    }
}

__global__ __launch_bounds__(64) void m2l_mfma_kernel(const float *__restrict__ W, float *__restrict__ V,
                                                      const float *__restrict__ ktab,
                                                      const uint32_t *__restrict__ tile_box,
                                                      const uint32_t *__restrict__ fpos,
                                                      const int32_t *__restrict__ slot_oi, TileBase tb, int64_t ngroups) {
    // Virtual block v = 8 * group + class: the eight parity classes of one group of 4 x 256
    // consecutive boxes run back to back, so that the waves in flight share their far
    // partners in L2; hardware blocks go to the 8 XCDs round-robin, so XCD x takes the
    // contiguous range v in [x * ngroups, (x+1) * ngroups).
    const int64_t bi = block_index2();
    if ((bi >> 3) >= ngroups) return;
    const int64_t v = (bi & 7) * ngroups + (bi >> 3);
    const int par = (int)(v & 7);
    const int64_t tile0 = (int64_t)tb.b[par] + (v >> 3) * M2L_GROUP;   // classes hold whole groups of tiles
    if (tile0 >= (int64_t)tb.b[par + 1]) return;
    const int lane = threadIdx.x;
    const int n = lane & 31, h = lane >> 5;
    const int32_t *soi = slot_oi + par * M2L_NSLOT;
    const float4 *ktab4 = reinterpret_cast<const float4 *>(ktab);
    const uint32_t *fp = fpos + tile0 * (int64_t)(M2L_NSLOT * M2L_TILE) + n;
    f16v a00 = {0.f}, a01 = {0.f}, a10 = {0.f}, a11 = {0.f}, a20 = {0.f}, a21 = {0.f}, a30 = {0.f}, a31 = {0.f};
    // far partners of slot 0; those of slot s+1 are fetched while slot s is multiplied
    uint32_t src[M2L_GROUP];
#pragma unroll
    for (int t = 0; t < M2L_GROUP; ++t) src[t] = fp[(int64_t)t * (M2L_NSLOT * M2L_TILE)];
#pragma unroll 1
    for (int s = 0; s < M2L_NSLOT; ++s) {
        const int oi = __builtin_amdgcn_readfirstlane(soi[s]);
        uint32_t nxt[M2L_GROUP];
        const int sn = s + 1 < M2L_NSLOT ? s + 1 : s;
#pragma unroll
        for (int t = 0; t < M2L_GROUP; ++t) nxt[t] = fp[(int64_t)t * (M2L_NSLOT * M2L_TILE) + sn * M2L_TILE];
        const float4 *Ap = ktab4 + (int64_t)oi * (M2L_R * M2L_R / 4) + lane;
        float4 A[16];
#pragma unroll
        for (int g = 0; g < 16; ++g) A[g] = Ap[g * 64];
        m2l_tile(W, src[0], h, A, a00, a01);
        m2l_tile(W, src[1], h, A, a10, a11);
        m2l_tile(W, src[2], h, A, a20, a21);
        m2l_tile(W, src[3], h, A, a30, a31);
#pragma unroll
        for (int t = 0; t < M2L_GROUP; ++t) src[t] = nxt[t];
    }
    const uint32_t *tb4 = tile_box + tile0 * M2L_TILE + n;
    m2l_store(V, tb4[0 * M2L_TILE], h, a00, a01);
    m2l_store(V, tb4[1 * M2L_TILE], h, a10, a11);
    m2l_store(V, tb4[2 * M2L_TILE], h, a20, a21);
    m2l_store(V, tb4[3 * M2L_TILE], h, a30, a31);
}

bool m2l_tables_apply(const f3m_plan_s &P) { return P.D == 3 && P.p == 4 && P.T == 4 && !P.force_all_near; }

void m2l_prepare_plan(f3m_plan_s &P, hipStream_t st) {
    std::vector<int32_t> so, soi;
    make_slot_tables(so, soi);
    P.slot_of.alloc(so.size(), &P.bytes);
    P.slot_oi.alloc(soi.size(), &P.bytes);
    F3M_HIP(hipMemcpyAsync(P.slot_of.p, so.data(), so.size() * sizeof(int32_t), hipMemcpyHostToDevice, st));
    F3M_HIP(hipMemcpyAsync(P.slot_oi.p, soi.data(), soi.size() * sizeof(int32_t), hipMemcpyHostToDevice, st));
    F3M_HIP(hipStreamSynchronize(st));
}

// Everything the table-driven M2L of one depth needs except the far partners themselves,
// which the list kernel writes into fpos afterwards.
void m2l_prepare_level(f3m_plan_s &P, int level, hipStream_t st) {
    f3m_level &lv = P.lev[level];
    int64_t *tally = &P.bytes;
    NodeD nd;
    for (int i = 0; i < 4; ++i) nd.s[i] = std::cos((double)i * M_PI / 3.0);
    // kernel matrices of this depth
    const double half = 0.5 * (double)P.E / std::ldexp(1.0, level);
    const double c = half * half / (2.0 * (double)P.gamma * (double)P.gamma);
    const int64_t nk = (int64_t)M2L_NOFF * M2L_R * M2L_R;
    lv.ktab.alloc((size_t)nk, tally);
    ktab_kernel<<<dim3((unsigned)cdiv(nk, 256)), dim3(256), 0, st>>>(lv.ktab.p, nd, c);
    F3M_HIP(hipGetLastError());
    // tiles: the boxes of each parity class, in rank order, 32 per tile, whole groups per class
    lv.gpos.alloc((size_t)lv.nb);
    int64_t tiles = 0;
    std::vector<ScanState> S(8);
    for (uint32_t cidx = 0; cidx < 8; ++cidx) {
        scan_prepare(ParityIn{lv.key.p, cidx}, lv.nb, S[cidx], true, st);
        lv.tile_base[cidx] = (uint32_t)tiles;
        tiles += cdiv(cdiv((int64_t)S[cidx].total, M2L_TILE), M2L_GROUP) * M2L_GROUP;
    }
    lv.tile_base[8] = (uint32_t)tiles;
    lv.ntiles = tiles;
    lv.tile_box.alloc((size_t)tiles * M2L_TILE, tally);
    F3M_HIP(hipMemsetAsync(lv.tile_box.p, 0xFF, (size_t)tiles * M2L_TILE * sizeof(uint32_t), st));
    for (uint32_t cidx = 0; cidx < 8; ++cidx)
        scan_finish(ParityIn{lv.key.p, cidx}, lv.nb, S[cidx],
                    ParityOut{lv.tile_box.p, lv.gpos.p, (uint64_t)lv.tile_base[cidx] * M2L_TILE}, st);
    const size_t nf = (size_t)lv.ntiles * M2L_NSLOT * M2L_TILE;
    lv.fpos.alloc(nf, tally);
    F3M_HIP(hipMemsetAsync(lv.fpos.p, 0xFF, nf * sizeof(uint32_t), st));
    F3M_HIP(hipStreamSynchronize(st));   // the scan states are released on return
    lv.m2l_tables = true;
}

struct FposPairsIn {
    const uint32_t *tile_box, *fpos, *start;
    __device__ uint64_t operator()(int64_t g) const {
        const uint32_t a = tile_box[g];
        if (a == 0xFFFFFFFFu) return 0;
        const uint32_t *row = fpos + (g >> 5) * (int64_t)(M2L_NSLOT * M2L_TILE) + (g & 31);
        uint64_t s = 0;
        for (int k = 0; k < M2L_NSLOT; ++k) {
            const uint32_t q = row[(int64_t)k * M2L_TILE];
            if (q != 0xFFFFFFFFu) s += start[q + 1] - start[q];
        }
        return s * (uint64_t)(start[a + 1] - start[a]);
    }
};

int64_t m2l_far_point_pairs(const f3m_plan_s &P, int level, hipStream_t st) {
    const f3m_level &lv = P.lev[level];
    ScanState S;
    scan_prepare(FposPairsIn{lv.tile_box.p, lv.fpos.p, lv.start.p}, lv.ntiles * M2L_TILE, S, true, st);
    return (int64_t)S.total;
}

void m2l_materialize_far(const f3m_plan_s &P, int level, uint32_t *cols_dev, hipStream_t st) {
    const f3m_level &lv = P.lev[level];
    DevBuf<uint32_t> gpos;
    gpos.alloc((size_t)lv.nb);
    const int64_t nlanes = lv.ntiles * M2L_TILE;
    gpos_kernel<<<grid2(cdiv(nlanes, 256)), dim3(256), 0, st>>>(lv.tile_box.p, nlanes, gpos.p);
    far_rows_kernel<<<grid2(cdiv(lv.nb, 64)), dim3(64), 0, st>>>(gpos.p, lv.nb, lv.far_ptr.p, lv.fpos.p, cols_dev);
    F3M_HIP(hipGetLastError());
    F3M_HIP(hipStreamSynchronize(st));
}

bool run_m2l_tables(f3m_plan_s &P, int level, const float *W, float *V, hipStream_t st) {
    f3m_level &lv = P.lev[level];
    if (!lv.m2l_tables) return false;
    TileBase tb;
    for (int c = 0; c < 9; ++c) tb.b[c] = lv.tile_base[c];
    int64_t ngroups = 0;   // blocks of the largest class
    for (int c = 0; c < 8; ++c) ngroups = std::max<int64_t>(ngroups, (lv.tile_base[c + 1] - lv.tile_base[c]) / M2L_GROUP);
    m2l_mfma_kernel<<<grid2(ngroups * 8), dim3(64), 0, st>>>(W, V, lv.ktab.p, lv.tile_box.p,
                                                                         lv.fpos.p, P.slot_oi.p, tb, ngroups);
    F3M_HIP(hipGetLastError());
    return true;
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

template <int CTRL>
__device__ inline float dpp_quad(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

__global__ __launch_bounds__(512) void m2l_stencil_kernel(const uint64_t *__restrict__ up_near_ptr,
                                                          const uint32_t *__restrict__ up_near_col,
                                                          const uint32_t *__restrict__ up_cstart,
                                                          const int32_t *__restrict__ up_cell,
                                                          const int32_t *__restrict__ cell,
                                                          const uint32_t *__restrict__ key, int64_t nparents,
                                                          int64_t per_xcd, const float *__restrict__ G,
                                                          const float *__restrict__ W, float *__restrict__ V) {
    __shared__ float rows[ST_CAND * 64];
    __shared__ int present[ST_CAND];
    __shared__ uint32_t cand[ST_CAND];      // candidate k of near parent j at [8 j + k]: rank or ~0
    __shared__ int cpos[ST_CAND];           // its position in the 6 x 6 x 6 grid
    __shared__ uint32_t qfirst[27], qcount[27];
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
    // far and present candidates, one bit each
    uint64_t mask[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int m = lane + 64 * k;
        bool ok = false;
        if (m < ST_CAND) {
            const int ox = m % 6 - 2 - tx, oy = (m / 6) % 6 - 2 - ty, oz = m / 36 - 2 - tz;
            ok = present[m] != 0 && ox * ox + oy * oy + oz * oz >= 4;
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
            fx[c][k] = G[(c + 1 - tx) * 16 + ix * 4 + ((ix + k) & 3)];
            fy[c][k] = G[(c + 1 - ty) * 16 + iy * 4 + ((iy + k) & 3)];
            fz[c][k] = G[(c + 1 - tz) * 16 + iz * 4 + ((iz + k) & 3)];
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
#pragma unroll
            for (int cx = 0; cx < 6; ++cx) {
                const int m = cx + 6 * cy + 36 * cz;
                if ((mask[m >> 6] >> (m & 63)) & 1ull) {
                    // line += sum_k fx[cx][k] * (entry k places further in the lane's quad); the
                    // row value comes straight from the LDS read, so no vector-ALU write
                    // precedes the DPP reads of it
                    asm("v_fmac_f32 %0, %2, %1\n\t"
                        "v_fmac_f32_dpp %0, %1, %3 quad_perm:[1,2,3,0] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                        "v_fmac_f32_dpp %0, %1, %4 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
                        "v_fmac_f32_dpp %0, %1, %5 quad_perm:[3,0,1,2] row_mask:0xf bank_mask:0xf bound_ctrl:1"
                        : "+v"(line)
                        : "v"(v[cx]), "v"(fx[cx][0]), "v"(fx[cx][1]), "v"(fx[cx][2]), "v"(fx[cx][3]));
                }
            }
            plane = fmaf(fy[cy][0], line, plane);
#pragma unroll
            for (int k = 1; k < 4; ++k) plane = fmaf(fy[cy][k], __shfl(line, ylane[k], 64), plane);
        }
        acc = fmaf(fz[cz][0], plane, acc);
#pragma unroll
        for (int k = 1; k < 4; ++k) acc = fmaf(fz[cz][k], __shfl(plane, zlane[k], 64), acc);
    }
    V[(int64_t)t * 64 + lane] = acc;
}

bool run_m2l_stencil(f3m_plan_s &P, int level, const float *W, float *V, hipStream_t st) {
    if (!m2l_tables_apply(P) || level < 1) return false;
    f3m_level &lv = P.lev[level], &up = P.lev[level - 1];
    if (lv.gtab.p == nullptr || lv.gtab_omax != 3) return false;
    const int64_t per_xcd = cdiv(up.nb, 8);
    m2l_stencil_kernel<<<grid2(per_xcd * 8), dim3(512), 0, st>>>(up.near_ptr.p, up.near_col.p, up.cstart.p, up.cell.p,
                                                                lv.cell.p, lv.key.p, up.nb, per_xcd, lv.gtab.p, W, V);
    F3M_HIP(hipGetLastError());
    return true;
}

}  // namespace f3m
