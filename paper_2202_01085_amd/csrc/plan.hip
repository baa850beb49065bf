// f3m_plan: enclosing cube, keys, radix sort, box tables, interaction lists.
// (arXiv 2202.01085: Sec. 3 "Enclosing and partitioning the data", Sec. 4.1, Sec. 4.2,
//  Appendix E Algorithm 1 "Divide", "Calculate interactions left", "Partition".)
#include <algorithm>
#include <cmath>
#include <cstring>

#include "plan.h"

f3m_plan_s::~f3m_plan_s() {
    for (auto &e : ev)
        if (e) (void)hipEventDestroy(e);
    for (auto &e : far_events)
        if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : {ev_fork, ev_join, ev_p2p0, ev_p2p1})
        if (e) (void)hipEventDestroy(e);
    if (side) (void)hipStreamDestroy(side);
}

namespace f3m {

int quant_depth(int D) {
    int q = 32 / D;
    return q > 20 ? 20 : q;
}

// ------------------------------------------------------------------------------------
// enclosing cube: per-dimension min and max (exact in fp32), non-finite detection
// ------------------------------------------------------------------------------------
constexpr int BBOX_BLOCKS = 1024;
constexpr int BBOX_NT = 256;

template <int D>
__global__ __launch_bounds__(BBOX_NT) void bbox_kernel(const float *__restrict__ X, int64_t n,
                                                       float *__restrict__ part, int *__restrict__ nonfinite) {
    float mn[D], mx[D];
#pragma unroll
    for (int d = 0; d < D; ++d) { mn[d] = INFINITY; mx[d] = -INFINITY; }
    int bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * BBOX_NT + threadIdx.x; i < n; i += (int64_t)gridDim.x * BBOX_NT) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            float v = X[i * D + d];
            bad |= !(fabsf(v) <= 3.402823466e38f);
            mn[d] = fminf(mn[d], v);
            mx[d] = fmaxf(mx[d], v);
        }
    }
    __shared__ float smn[BBOX_NT / 64][D], smx[BBOX_NT / 64][D];
    __shared__ int sbad;
    if (threadIdx.x == 0) sbad = 0;
    __syncthreads();
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
    for (int d = 0; d < D; ++d) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            mn[d] = fminf(mn[d], __shfl_xor(mn[d], off, 64));
            mx[d] = fmaxf(mx[d], __shfl_xor(mx[d], off, 64));
        }
        if (lane == 0) { smn[w][d] = mn[d]; smx[w][d] = mx[d]; }
    }
    if (bad) atomicOr(&sbad, 1);
    __syncthreads();
    if (threadIdx.x < D) {
        int d = threadIdx.x;
        float a = smn[0][d], b = smx[0][d];
        for (int k = 1; k < BBOX_NT / 64; ++k) { a = fminf(a, smn[k][d]); b = fmaxf(b, smx[k][d]); }
        part[(int64_t)blockIdx.x * 2 * D + d] = a;
        part[(int64_t)blockIdx.x * 2 * D + D + d] = b;
    }
    if (threadIdx.x == 0 && sbad) atomicOr(nonfinite, 1);
}

// ------------------------------------------------------------------------------------
// cells and keys (Sec. 4.2 box-index formula).  The cell of a point is fixed once, at the
// quantisation depth Lq, by two separately rounded fp32 operations and a truncation:
//   c_d = min( trunc( (x_d - alpha_d) * s ), 2^Lq - 1 ),   s = fl32(2^Lq / E)
// The cell at depth l is c_d >> (Lq - l).  Key: bit k of c_d -> key bit k*D + d.
// ------------------------------------------------------------------------------------
struct AlphaArg { float a[F3M_MAX_DIM]; };

// bit k of c -> bit k * D (c < 2^(32 / D))
template <int D>
__device__ inline uint32_t spread_bits(uint32_t c) {
    if constexpr (D == 1) {
        return c;
    } else if constexpr (D == 2) {
        c &= 0xFFFFu;
        c = (c | (c << 8)) & 0x00FF00FFu;
        c = (c | (c << 4)) & 0x0F0F0F0Fu;
        c = (c | (c << 2)) & 0x33333333u;
        return (c | (c << 1)) & 0x55555555u;
    } else if constexpr (D == 3) {
        c &= 0x3FFu;
        c = (c | (c << 16)) & 0x030000FFu;
        c = (c | (c << 8)) & 0x0300F00Fu;
        c = (c | (c << 4)) & 0x030C30C3u;
        return (c | (c << 2)) & 0x09249249u;
    } else {
        uint32_t r = 0;
#pragma unroll
        for (int k = 0; k < 32 / D; ++k) r |= ((c >> k) & 1u) << (k * D);
        return r;
    }
}

template <int D>
__global__ __launch_bounds__(256) void keys_kernel(const float *__restrict__ X, int64_t n, AlphaArg alpha, float s,
                                                   int Lq, uint32_t *__restrict__ keys) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    uint32_t cmax = (uint32_t)((1ull << Lq) - 1);
    uint32_t key = 0;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        float diff = __fsub_rn(X[i * D + d], alpha.a[d]);
        float u = __fmul_rn(diff, s);
        uint32_t c = (uint32_t)u;
        c = c > cmax ? cmax : c;
        key |= spread_bits<D>(c) << d;   // c < 2^Lq and Lq * D <= 32
    }
    keys[i] = key;
}

// ------------------------------------------------------------------------------------
// stable LSD radix sort of (key, index) pairs, 8 bits per pass:
//   histogram per tile -> exclusive scan in digit-major order -> stable scatter.
// This replaces the count / cumulative-sum / atomic-increment grouping of Sec. 4.1: the
// result is deterministic (ascending key, then ascending original index).
// ------------------------------------------------------------------------------------
constexpr int RS_NT = 256;
constexpr int RS_IPT = 32;
constexpr int RS_TILE = RS_NT * RS_IPT;

__global__ __launch_bounds__(RS_NT) void rs_hist_kernel(const uint32_t *__restrict__ keys, int64_t n, int shift,
                                                        uint32_t *__restrict__ hist, int64_t nblk) {
    __shared__ uint32_t h[256];
    // tiles are dealt to the dies like those of the scatter kernel (the counts of neighbouring tiles share lines)
    const int64_t per_die = (nblk + 7) / 8;
    const int64_t tile = (int64_t)(blockIdx.x & 7u) * per_die + (blockIdx.x >> 3);
    if (tile >= nblk) return;
    h[threadIdx.x] = 0;
    __syncthreads();
    // all loads first, four keys each, without a bounds test (the key buffers carry a tile of slack behind the
    // last key); what lies behind the end is left out of the counts
    const int64_t base = tile * RS_TILE;
    const int64_t left = n - base;
    const int cntile = (int)(left < RS_TILE ? left : RS_TILE);
    const uint4 *kp = reinterpret_cast<const uint4 *>(keys + base);
    uint4 v[RS_IPT / 4];
#pragma unroll
    for (int k = 0; k < RS_IPT / 4; ++k) v[k] = kp[k * RS_NT + threadIdx.x];
#pragma unroll
    for (int k = 0; k < RS_IPT / 4; ++k) {
        const int i0 = (k * RS_NT + (int)threadIdx.x) * 4;
        const uint32_t key4[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (i0 + c < cntile) atomicAdd(&h[(key4[c] >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * nblk + tile] = h[threadIdx.x];
}

struct U32In {
    const uint32_t *p;
    __device__ uint64_t operator()(int64_t i) const { return p[i]; }
};
struct U32Out {
    uint32_t *p;
    __device__ void operator()(int64_t i, uint64_t ex, uint64_t) const { p[i] = (uint32_t)ex; }
};

// Stable scatter of one tile of RS_TILE keys.  Tile order = (wave, round, lane): every wave
// ranks its own 32 rounds of 64 keys with a private LDS counter array, with no block barrier
// inside the loop; then the tile is put in digit order in LDS and written out so that
// consecutive threads write consecutive addresses of a digit run.  The buffers must be readable
// for a whole tile behind the last key.
template <bool FIRST>   // FIRST: the values are the positions themselves (vals_in is not read)
__global__ __launch_bounds__(RS_NT, 4) void rs_scatter_kernel(const uint32_t *__restrict__ keys_in,
                                                           const uint32_t *__restrict__ vals_in,
                                                           uint32_t *__restrict__ keys_out,
                                                           uint32_t *__restrict__ vals_out, int64_t n, int shift,
                                                           const uint32_t *__restrict__ offs, int64_t nblk) {
    constexpr int NW = RS_NT / 64;
    __shared__ uint32_t wcnt[NW][256];      // per wave: keys of each digit seen so far
    __shared__ uint32_t dstart[256];        // first tile-local position of each digit
    __shared__ uint32_t gbase[256];         // global position of the tile's first key of each digit
    __shared__ __attribute__((aligned(8))) uint32_t sbuf[RS_TILE];   // the tile in digit order: first its keys, then its values
    // per wave, while the keys are ranked (sbuf is not in use yet): the lanes that hold each digit in the current round
    uint64_t (*wmask)[256] = reinterpret_cast<uint64_t (*)[256]>(sbuf);
    static_assert(sizeof(uint64_t) * NW * 256 <= sizeof(uint32_t) * RS_TILE, "the lane masks must fit the tile buffer");
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    // Workgroups go to the 8 dies in turn; every die takes a contiguous range of tiles, so that the runs
    // which neighbouring tiles append to the same digit meet in one L2 and leave it as whole lines.
    const int64_t per_die = (nblk + 7) / 8;
    const int64_t tile = (int64_t)(blockIdx.x & 7u) * per_die + (blockIdx.x >> 3);
    if (tile >= nblk) return;
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        wcnt[k][tid] = 0;
        wmask[k][tid] = 0ull;
    }
    gbase[tid] = offs[(int64_t)tid * nblk + tile];
    __syncthreads();
    const int64_t base = tile * RS_TILE + (int64_t)w * (RS_IPT * 64);
    // Registers are what bounds the number of resident workgroups: ranks and positions are kept as 16-bit
    // halves (a tile has 8192 places; 0xFFFF = out of range), the digits of the written keys as bytes.
    uint32_t key[RS_IPT], val[RS_IPT], rk[RS_IPT / 2];
    const int64_t left = n - tile * RS_TILE;
    const int cntile = (int)(left < RS_TILE ? left : RS_TILE);   // keys of this tile (the last one may be short)
    const int local = w * (RS_IPT * 64) + lane;                  // tile-local index of this thread's first key
    // loads without branches: the buffers carry a tile of slack, and what is read behind the end is left out of
    // the ranking below
    const uint32_t *kp = keys_in + base + lane, *vp = vals_in + base + lane;
#pragma unroll
    for (int r = 0; r < RS_IPT; ++r) key[r] = kp[r * 64];
    // Rank of a key among the earlier keys of its wave with the same digit.  The lanes of a round that hold the
    // same digit find each other through LDS: every lane ORs its own bit into the 64-bit word of its digit
    // (an atomic OR: the result does not depend on the order), reads the word back, and counts the bits below
    // its own.  The first lane of each group then adds the group to the running count of the digit and clears
    // the word.  (LDS operations of a wave complete in order, and the wave runs in lockstep.)
    const uint64_t mybit = 1ull << lane;
#pragma unroll
    for (int r = 0; r < RS_IPT; ++r) {
        const bool valid = local + r * 64 < cntile;
        const uint32_t digit = (key[r] >> shift) & 255u;
        uint32_t rank = 0xFFFFu;
        if (valid) {
            atomicOr(reinterpret_cast<unsigned long long *>(&wmask[w][digit]), (unsigned long long)mybit);
            __builtin_amdgcn_wave_barrier();
            const uint64_t peers = wmask[w][digit];
            const uint32_t cnt = wcnt[w][digit];
            const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
            rank = cnt + before;   // within (wave, digit): below 2048
            __builtin_amdgcn_wave_barrier();
            if (before == 0) {
                wcnt[w][digit] = cnt + (uint32_t)__popcll(peers);
                wmask[w][digit] = 0ull;
            }
        }
        rk[r >> 1] = (r & 1) ? (rk[r >> 1] | (rank << 16)) : rank;
        __builtin_amdgcn_wave_barrier();   // keep the rounds' LDS accesses in program order
    }
    __syncthreads();
    // digit totals of the tile, exclusive scan over the 256 digits (one digit per thread)
    {
        uint32_t tot = 0;
#pragma unroll
        for (int k = 0; k < NW; ++k) tot += wcnt[k][tid];
        uint64_t blocktot;
        const uint32_t ex = (uint32_t)block_excl_scan_u64(tot, &blocktot);
        dstart[tid] = ex;
    }
    __syncthreads();
    // keys and values pass through the same 32 KB of LDS one after the other
#pragma unroll
    for (int r = 0; r < RS_IPT; ++r) {
        const uint32_t rank = (rk[r >> 1] >> (16 * (r & 1))) & 0xFFFFu;
        if (rank != 0xFFFFu) {
            const uint32_t digit = (key[r] >> shift) & 255u;
            uint32_t pos = dstart[digit] + rank;
            for (int k = 0; k < w; ++k) pos += wcnt[k][digit];
            rk[r >> 1] = (r & 1) ? ((rk[r >> 1] & 0xFFFFu) | (pos << 16)) : ((rk[r >> 1] & 0xFFFF0000u) | pos);
            sbuf[pos] = key[r];
        }
    }
    // the values are loaded only now, into the registers of the keys (keys, values and ranks together would not
    // fit the register budget of four workgroups per compute unit); they arrive while the keys are written out
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int r = 0; r < RS_IPT; ++r) {
        if constexpr (FIRST) val[r] = (uint32_t)(base + r * 64 + lane);
        else val[r] = vp[r * 64];
    }
    __syncthreads();
    uint32_t dig[RS_IPT / 4];   // digit of the tile's entry r * RS_NT + tid
#pragma unroll
    for (int r = 0; r < RS_IPT; ++r) {
        const int pos = r * RS_NT + tid;
        uint32_t digit = 0;
        if (pos < cntile) {
            const uint32_t k = sbuf[pos];
            digit = (k >> shift) & 255u;
            keys_out[gbase[digit] + ((uint32_t)pos - dstart[digit])] = k;
        }
        dig[r >> 2] = (r & 3) ? (dig[r >> 2] | (digit << (8 * (r & 3)))) : digit;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RS_IPT; ++r) {
        const uint32_t pos = (rk[r >> 1] >> (16 * (r & 1))) & 0xFFFFu;
        if (pos != 0xFFFFu) sbuf[pos] = val[r];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RS_IPT; ++r) {
        const int pos = r * RS_NT + tid;
        if (pos < cntile) {
            const uint32_t digit = (dig[r >> 2] >> (8 * (r & 3))) & 255u;
            vals_out[gbase[digit] + ((uint32_t)pos - dstart[digit])] = sbuf[pos];
        }
    }
}

// sorts (keys_a, index) by the low `bits` bits; returns true if the result is in the b buffers
static bool radix_sort(uint32_t *keys_a, uint32_t *vals_a, uint32_t *keys_b, uint32_t *vals_b, int64_t n, int bits,
                       hipStream_t st) {
    int64_t nblk = cdiv(n, RS_TILE);
    DevBuf<uint32_t> hist;
    hist.alloc((size_t)nblk * 256);
    bool in_b = false, first = true;
    for (int shift = 0; shift < bits; shift += 8) {
        const uint32_t *kin = in_b ? keys_b : keys_a;
        const uint32_t *vin = first ? nullptr : (in_b ? vals_b : vals_a);
        uint32_t *kout = in_b ? keys_a : keys_b;
        uint32_t *vout = in_b ? vals_a : vals_b;
        rs_hist_kernel<<<dim3((unsigned)((nblk + 7) / 8 * 8)), dim3(RS_NT), 0, st>>>(kin, n, shift, hist.p, nblk);
        F3M_HIP(hipGetLastError());
        exclusive_scan(U32In{hist.p}, nblk * 256, U32Out{hist.p}, nullptr, st);
        const unsigned grid = (unsigned)((nblk + 7) / 8 * 8);   // a whole number of rounds over the dies
        if (first)
            rs_scatter_kernel<true><<<dim3(grid), dim3(RS_NT), 0, st>>>(kin, vin, kout, vout, n, shift, hist.p, nblk);
        else
            rs_scatter_kernel<false><<<dim3(grid), dim3(RS_NT), 0, st>>>(kin, vin, kout, vout, n, shift, hist.p, nblk);
        F3M_HIP(hipGetLastError());
        in_b = !in_b;
        first = false;
    }
    F3M_HIP(hipStreamSynchronize(st));
    return in_b;
}

__global__ void iota_kernel(uint32_t *p, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = (uint32_t)i;
}

template <int D>
__global__ __launch_bounds__(256) void gather_rows_kernel(const float *__restrict__ X, const uint32_t *__restrict__ perm,
                                                          int64_t n, float *__restrict__ Xs) {
    int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= n) return;
    int64_t j = perm[k];
#pragma unroll
    for (int d = 0; d < D; ++d) Xs[k * D + d] = X[j * D + d];
}

// ------------------------------------------------------------------------------------
// box tables per depth (Algorithm 1 "Divide"; empty boxes never appear, Sec. 4.2)
// ------------------------------------------------------------------------------------
struct HeadIn {
    const uint32_t *keys;
    int shift;
    __device__ uint64_t operator()(int64_t i) const {
        if (i == 0) return 1;
        return ((uint64_t)keys[i] >> shift) != ((uint64_t)keys[i - 1] >> shift);
    }
    // a run of 8 keys (base a multiple of 8, so 32-byte aligned: the arrays come from the pool) in two loads
    __device__ void load_run(int64_t base, uint64_t (&v)[SCAN_IPT]) const {
        static_assert(SCAN_IPT == 8, "two loads of four keys");
        const uint4 *p = reinterpret_cast<const uint4 *>(keys + base);
        const uint4 a = p[0], b = p[1];
        const uint32_t k[9] = {base > 0 ? keys[base - 1] : 0u, a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = ((uint64_t)k[j + 1] >> shift) != ((uint64_t)k[j] >> shift);
        if (base == 0) v[0] = 1;
    }
};
struct HeadOut {
    const uint32_t *keys;
    int shift;
    uint32_t *start, *bkey;
    __device__ void operator()(int64_t i, uint64_t ex, uint64_t v) const {
        if (v) {
            start[ex] = (uint32_t)i;
            bkey[ex] = (uint32_t)((uint64_t)keys[i] >> shift);
        }
    }
};
struct ParentOut {
    uint32_t *parent, *cstart_up;
    __device__ void operator()(int64_t a, uint64_t ex, uint64_t v) const {
        parent[a] = (uint32_t)(ex + v - 1);
        if (v) cstart_up[ex] = (uint32_t)a;
    }
};

// Divide from the depth above (used while boxes are much fewer than points): the children of a
// box are sub-intervals of its sorted interval, found by binary search on the key prefix.
// lb[P * 2^D + c] = first point of parent P whose depth-l key is >= (key_P << D | c).
template <int D>
__global__ __launch_bounds__(256) void child_bounds_kernel(const uint32_t *__restrict__ keys, int shift,
                                                           const uint32_t *__restrict__ up_start, int64_t nslots,
                                                           const uint32_t *__restrict__ up_key, uint32_t *__restrict__ lb) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= nslots) return;
    const int64_t P = idx >> D;
    const uint32_t c = (uint32_t)(idx & ((1 << D) - 1));
    uint32_t lo = up_start[P], hi = up_start[P + 1];
    if (c != 0) {
        const uint64_t want = ((uint64_t)up_key[P] << D) | c;
        while (lo < hi) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            if (((uint64_t)keys[mid] >> shift) < want) lo = mid + 1;
            else hi = mid;
        }
    }
    lb[idx] = lo;
}
struct ChildIn {
    const uint32_t *lb;   // [nslots + 1]
    __device__ uint64_t operator()(int64_t i) const { return lb[i + 1] != lb[i]; }
};
template <int D>
struct ChildOut {
    const uint32_t *lb, *up_key;
    uint32_t *start, *bkey, *parent, *cstart_up;
    __device__ void operator()(int64_t i, uint64_t ex, uint64_t v) const {
        const int64_t P = i >> D;
        const uint32_t c = (uint32_t)(i & ((1 << D) - 1));
        if (c == 0) cstart_up[P] = (uint32_t)ex;
        if (v) {
            start[ex] = lb[i];
            bkey[ex] = (uint32_t)(((uint64_t)up_key[P] << D) | c);
            parent[ex] = (uint32_t)P;
        }
    }
};

__global__ void set_u32_kernel(uint32_t *p, uint32_t v) { *p = v; }
__global__ void set_u64_kernel(uint64_t *p, uint64_t v) { *p = v; }

__global__ __launch_bounds__(256) void max_count_kernel(const uint32_t *__restrict__ start, int64_t nb,
                                                        uint32_t *__restrict__ part) {
    uint32_t m = 0;
    for (int64_t a = (int64_t)blockIdx.x * 256 + threadIdx.x; a < nb; a += (int64_t)gridDim.x * 256)
        m = max(m, start[a + 1] - start[a]);
    __shared__ uint32_t sm[256];
    sm[threadIdx.x] = m;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) sm[threadIdx.x] = max(sm[threadIdx.x], sm[threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = sm[0];
}

template <int D>
__global__ __launch_bounds__(256) void cells_kernel(const uint32_t *__restrict__ bkey, int64_t nb, int level,
                                                    int32_t *__restrict__ cell) {
    int64_t a = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (a >= nb) return;
    uint32_t key = bkey[a];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        int32_t c = 0;
        for (int k = 0; k < level; ++k) c |= (int32_t)((key >> (k * D + d)) & 1u) << k;
        cell[a * D + d] = c;
    }
}

// ------------------------------------------------------------------------------------
// interaction lists (Algorithm 1 "Calculate interactions left" and "Partition"):
// the candidates of a box are the children of the boxes near its parent; a candidate is
// far iff the squared integer cell offset is >= T = ceil(theta^2)  (Sec. 3, IsFarField
// := |delta centre| >= 2 l, divided by l).  Rows come out sorted by column rank because the
// parent's row is sorted and children have consecutive ranks (Sec. 4.1 "Ensuring
// interactions are sorted").  pass 0 counts, pass 1 fills.  A null near_col or far_col skips
// that side: depths whose M2L works on the candidate grid keep only the far counts, and their
// far rows are produced on request.
// ------------------------------------------------------------------------------------
struct ListArg {
    int T;                 // a pair is far iff the squared integer cell offset is >= T
    int mode;              // 0: far rule, 1: all near, 2: all far (smooth depth, Sec. 4.3)
    uint32_t rho;          // small field (Sec. 4.2): |p| + |q| <= rho goes on the direct list; 0 = off
    const uint32_t *start; // point intervals of the target boxes of this depth (sizes for the small-field rule)
    // source side of the depth: the same tables as the targets' for one point set, those of Y for two
    const int32_t *cell_src;
    const uint32_t *start_src;
    // two sets: the grids are shifted by u box edges, and a pair is far iff
    // sum_d ((c'_d - c_d) + u_d)^2 >= theta2, every fp64 operation rounded on its own, d ascending
    int shifted;
    double u[F3M_MAX_DIM];
    double theta2;
    uint32_t *cnt_near, *cnt_far, *cnt_small;         // pass 0: row lengths
    const uint64_t *near_ptr, *far_ptr, *small_ptr;   // pass 1: row offsets
    uint32_t *near_col, *far_col, *small_col;         // pass 1: columns (null: that list is not written)
    // pass 1 of the by-parent kernel, D = 3, far ratio 2: the tables of the candidate-grid M2L (or null):
    // [parent][216] rank of the candidate at each position of the 6 x 6 x 6 grid around the parent,
    // [parent][8] the child of each parity (both preset to ~0)
    uint32_t *st_cand, *st_child;
};

// up_cstart: children intervals of the SOURCE-side boxes one depth up
template <int D>
__global__ __launch_bounds__(128) void lists_kernel(int pass, int64_t nb, const uint32_t *__restrict__ parent,
                                                    const int32_t *__restrict__ cell,
                                                    const uint64_t *__restrict__ up_near_ptr,
                                                    const uint32_t *__restrict__ up_near_col,
                                                    const uint32_t *__restrict__ up_cstart, ListArg A) {
    int64_t a = (int64_t)blockIdx.x * 128 + threadIdx.x;
    if (a >= nb) return;
    int32_t ca[D];
#pragma unroll
    for (int d = 0; d < D; ++d) ca[d] = cell[a * D + d];
    uint32_t P = parent[a];
    uint64_t nn = 0, nf = 0, ns = 0;
    const uint64_t nbase = pass && A.near_ptr ? A.near_ptr[a] : 0, fbase = pass && A.far_ptr ? A.far_ptr[a] : 0,
                   sbase = pass && A.small_ptr ? A.small_ptr[a] : 0;
    const uint32_t cnt_a = A.rho ? A.start[a + 1] - A.start[a] : 0u;
    for (uint64_t e = up_near_ptr[P]; e < up_near_ptr[P + 1]; ++e) {
        uint32_t Q = up_near_col[e];
        uint32_t b1 = up_cstart[Q + 1];
        for (uint32_t bq = up_cstart[Q]; bq < b1; ++bq) {
            int d2 = 0;
            int o[D];
#pragma unroll
            for (int d = 0; d < D; ++d) {
                o[d] = A.cell_src[(int64_t)bq * D + d] - ca[d];
                d2 += o[d] * o[d];
            }
            bool far_rule = d2 >= A.T;
            if (A.shifted) {
                double s = 0.0;
#pragma unroll
                for (int d = 0; d < D; ++d) {
                    const double t = __dadd_rn((double)o[d], A.u[d]);
                    s = __dadd_rn(s, __dmul_rn(t, t));
                }
                far_rule = s >= A.theta2;
            }
            const bool is_small = A.rho && A.mode != 1 && cnt_a + (A.start_src[bq + 1] - A.start_src[bq]) <= A.rho;
            const bool is_far = A.mode == 2 || (A.mode == 0 && far_rule);
            if (is_small) {
                if (pass && A.small_col) A.small_col[sbase + ns] = bq;
                ++ns;
            } else if (is_far) {
                if (pass && A.far_col) A.far_col[fbase + nf] = bq;
                ++nf;
            } else {
                if (pass && A.near_col) A.near_col[nbase + nn] = bq;
                ++nn;
            }
        }
    }
    if (!pass) {
        A.cnt_near[a] = (uint32_t)nn;
        A.cnt_far[a] = (uint32_t)nf;
        if (A.cnt_small) A.cnt_small[a] = (uint32_t)ns;
    }
}

// The same lists by parent (one point set, far rule only, D <= 3): the 2^D children of a parent
// share their candidates, so one wavefront per parent enumerates them once, 64 to a step with a lane
// per candidate, and tests them against every child.  The candidates of a round are the children
// of up to 64 boxes near the parent, written into LDS in sequence order (lane = near box, running
// sum of the child counts); ballots keep a child's near and far entries in that order.
template <int D>
__global__ __launch_bounds__(64) void lists_parent_kernel(int pass, int64_t nparents,
                                                          const uint32_t *__restrict__ cstart,
                                                          const int32_t *__restrict__ cell,
                                                          const uint64_t *__restrict__ up_near_ptr,
                                                          const uint32_t *__restrict__ up_near_col, ListArg A) {
    constexpr int NC = 1 << D;   // children of a box, at most
    __shared__ uint32_t cand[64 * NC];
    // workgroups go to the 8 dies in turn; every die takes a contiguous range of parents, whose rows and candidates
    // neighbour each other in memory (whole lines leave one L2, shared candidates are read into one L2)
    const int64_t per_die = (nparents + 7) >> 3;
    const int64_t P = (int64_t)(blockIdx.x & 7u) * per_die + (int64_t)(blockIdx.x >> 3);
    if (P >= nparents) return;
    const int lane = threadIdx.x;
    const uint32_t a0 = cstart[P];
    const int nt = min((int)(cstart[P + 1] - a0), NC);
    if (nt <= 0) return;   // (boxes are never empty: cannot happen)
    // lane t < nt holds the cell and the row offsets of child a0 + t
    const uint32_t at = a0 + (uint32_t)min(lane, nt - 1);
    int32_t tc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) tc[d] = cell[(int64_t)at * D + d];
    uint64_t nbase = 0, fbase = 0;
    if (pass && A.near_ptr) nbase = A.near_ptr[at];
    if (pass && A.far_ptr) fbase = A.far_ptr[at];
    uint32_t nn[NC], nf[NC];   // entries so far per child (wave-uniform)
#pragma unroll
    for (int t = 0; t < NC; ++t) nn[t] = nf[t] = 0;
    const uint64_t e0 = up_near_ptr[P], e1 = up_near_ptr[P + 1];
    for (uint64_t er = e0; er < e1; er += 64) {
        const int m = (int)(e1 - er < 64 ? e1 - er : 64);
        uint32_t b0 = 0, nq = 0;
        if (lane < m) {
            const uint32_t Q = up_near_col[er + lane];
            b0 = cstart[Q];
            nq = min(cstart[Q + 1] - b0, (uint32_t)NC);
        }
        const uint32_t cend = wave_incl_scan_u32(nq);   // inclusive running sum of the child counts over the lanes
        const uint32_t cbeg = cend - nq;
        const uint32_t S = __builtin_amdgcn_readlane(cend, 63);   // candidates of this round, <= 64 NC
        __syncthreads();   // the previous round has been read
        for (uint32_t j = 0; j < nq; ++j) cand[cbeg + j] = b0 + j;
        __syncthreads();
        for (uint32_t w0 = 0; w0 < S; w0 += 64) {
            const bool live = w0 + lane < S;
            const uint32_t bq = live ? cand[w0 + lane] : 0u;   // (a lane beyond the sequence reads box 0, unused)
            int32_t cc[D];
#pragma unroll
            for (int d = 0; d < D; ++d) cc[d] = A.cell_src[(int64_t)bq * D + d];
            if constexpr (D == 3) {
                if (pass && A.st_cand && live) {
                    // grid position of the candidate: its cell minus twice the parent's cell, plus 2 (a box near
                    // the parent is within one cell of it, so every coordinate lies in [0, 6))
                    int pos = 0, mul = 1;
                    bool inside = true;
#pragma unroll
                    for (int d = 0; d < D; ++d) {
                        const int q = cc[d] - 2 * (__builtin_amdgcn_readlane(tc[d], 0) >> 1) + 2;
                        inside = inside && q >= 0 && q < 6;
                        pos += q * mul;
                        mul *= 6;
                    }
                    if (inside) A.st_cand[P * 216 + pos] = bq;
                }
            }
#pragma unroll
            for (int t = 0; t < NC; ++t) {
                if (t < nt) {   // wave-uniform
                    int d2 = 0;
#pragma unroll
                    for (int d = 0; d < D; ++d) {
                        const int o = cc[d] - __builtin_amdgcn_readlane(tc[d], t);
                        d2 += o * o;
                    }
                    const bool is_far = d2 >= A.T;
                    const uint64_t mn = __ballot(live && !is_far), mf = __ballot(live && is_far);
                    if (pass) {
                        const uint64_t below = (1ull << lane) - 1ull;
                        if (A.near_col && live && !is_far) {
                            const uint64_t base = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(nbase >> 32), t) << 32) |
                                                  (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)nbase, t);
                            A.near_col[base + nn[t] + (uint32_t)__popcll(mn & below)] = bq;
                        }
                        if (A.far_col && live && is_far) {
                            const uint64_t base = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(fbase >> 32), t) << 32) |
                                                  (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)fbase, t);
                            A.far_col[base + nf[t] + (uint32_t)__popcll(mf & below)] = bq;
                        }
                    }
                    nn[t] += (uint32_t)__popcll(mn);
                    nf[t] += (uint32_t)__popcll(mf);
                }
            }
        }
    }
    if constexpr (D == 3) {
        if (pass && A.st_child && lane < nt)   // the child of each parity (bit d = upper half along dimension d)
            A.st_child[P * 8 + ((tc[0] & 1) | ((tc[1] & 1) << 1) | ((tc[2] & 1) << 2))] = a0 + (uint32_t)lane;
    }
    if (!pass) {
        uint32_t vn = 0, vf = 0;
#pragma unroll
        for (int t = 0; t < NC; ++t)
            if (lane == t) { vn = nn[t]; vf = nf[t]; }
        if (lane < nt) {
            A.cnt_near[a0 + lane] = vn;
            A.cnt_far[a0 + lane] = vf;
            if (A.cnt_small) A.cnt_small[a0 + lane] = 0u;
        }
    }
}

// the rule of the depth is the plain far rule on one point set: the lists can be built by parent
static bool lists_by_parent(const ListArg &A, int D) { return D <= 3 && !A.shifted && A.rho == 0 && A.mode == 0; }

// the rule part of a list kernel argument for one depth of a plan
static ListArg list_rules(const f3m_plan_s &P, int level) {
    const f3m_level &lv = P.lev[level], &sv = P.slev(level);
    ListArg A{};
    A.T = P.T;
    A.mode = P.force_all_near ? 1 : lv.smooth ? 2 : 0;
    A.rho = (uint32_t)P.rho;
    A.start = lv.start.p;
    A.cell_src = sv.cell.p;
    A.start_src = sv.start.p;
    A.shifted = P.src ? 1 : 0;
    P.grid_shift(level, A.u);
    A.theta2 = (double)P.theta * (double)P.theta;
    return A;
}

// point pairs of a CSR interaction list: |p| * sum of |q| over the row of p
struct NearPairsIn {
    const uint32_t *start, *start_src;   // point intervals of the target boxes / of the source boxes
    const uint64_t *near_ptr;
    const uint32_t *near_col;
    __device__ uint64_t operator()(int64_t a) const {
        uint64_t s = 0;
        for (uint64_t e = near_ptr[a]; e < near_ptr[a + 1]; ++e) {
            uint32_t q = near_col[e];
            s += start_src[q + 1] - start_src[q];
        }
        return s * (uint64_t)(start[a + 1] - start[a]);
    }
};

struct PtrOut {
    uint64_t *p;
    __device__ void operator()(int64_t i, uint64_t ex, uint64_t) const { p[i] = ex; }
};

// ------------------------------------------------------------------------------------
// work splits: runs of at most `chunk` points inside a box
// ------------------------------------------------------------------------------------
struct ChunkCountIn {
    const uint32_t *start;
    uint32_t chunk;
    __device__ uint64_t operator()(int64_t a) const { return (start[a + 1] - start[a] + chunk - 1) / chunk; }
};

__global__ __launch_bounds__(256) void chunk_box_kernel(const uint32_t *__restrict__ first, int64_t nb, int64_t nchunks,
                                                        uint32_t *__restrict__ chunk_box) {
    int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= nchunks) return;
    // largest a with first[a] <= c   (first is non-decreasing, first[nb] = nchunks > c)
    int64_t lo = 0, hi = nb;
    while (hi - lo > 1) {
        int64_t mid = (lo + hi) >> 1;
        if ((int64_t)first[mid] <= c) lo = mid; else hi = mid;
    }
    chunk_box[c] = (uint32_t)lo;
}

// runs of at most `chunk` points inside the boxes whose row of a CSR list is not empty
struct ChunkCountIfIn {
    const uint32_t *start;
    const uint64_t *row_ptr;
    uint32_t chunk;
    __device__ uint64_t operator()(int64_t a) const {
        return row_ptr[a + 1] > row_ptr[a] ? (start[a + 1] - start[a] + chunk - 1) / chunk : 0;
    }
};

// runs of at most `chunk` points inside the boxes that carry a flag
struct ChunkCountFlagIn {
    const uint32_t *start;
    const uint32_t *flag;
    uint32_t chunk;
    __device__ uint64_t operator()(int64_t a) const { return flag[a] ? (start[a + 1] - start[a] + chunk - 1) / chunk : 0; }
};

// Near-field tiles of the last depth.  A box is cut into runs of 64 targets; a last run of at most `ts`
// targets (the overflow of a box a little above 64 points, or a box with very few points) would leave
// most of a 64-wide tile idle, so it becomes an "overflow tile" for the kernel that puts the SOURCES on
// the lanes instead.  Big tiles: the full runs, and the last run if it has more than ts targets.
struct BigTileCountIn {
    const uint32_t *start;
    uint32_t ts;
    __device__ uint64_t operator()(int64_t a) const {
        const uint32_t cnt = start[a + 1] - start[a];
        return cnt / 64u + ((cnt & 63u) > ts ? 1u : 0u);
    }
};
struct OverflowTileCountIn {
    const uint32_t *start;
    uint32_t ts;
    __device__ uint64_t operator()(int64_t a) const {
        const uint32_t rem = (start[a + 1] - start[a]) & 63u;
        return rem >= 1u && rem <= ts ? 1u : 0u;
    }
};

// Pairs of leaf boxes for the paired near field: one thread per parent walks its children in rank order and
// pairs child i with child i + 1 when their cells differ in one dimension only (by one cell, being siblings),
// both first runs of targets are big tiles (64 targets, or more than ts) and both near rows have at most 32
// entries.  paired[a] = 1 for the first box of a pair, 2 for the second, 0 otherwise.
__global__ __launch_bounds__(256) void pair_flag_kernel(int64_t nparents, const uint32_t *__restrict__ cstart,
                                                        const int32_t *__restrict__ cell,
                                                        const uint32_t *__restrict__ start,
                                                        const uint64_t *__restrict__ near_ptr, uint32_t ts,
                                                        uint8_t *__restrict__ paired) {
    const int64_t P = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (P >= nparents) return;
    const uint32_t c0 = cstart[P], c1 = cstart[P + 1];
    auto fits = [&](uint32_t a) {
        const uint32_t cnt = start[a + 1] - start[a];
        return (cnt >= 64u || cnt > ts) && near_ptr[a + 1] - near_ptr[a] <= 32u;
    };
    uint32_t a = c0;
    while (a < c1) {
        bool pair = false;
        if (a + 1 < c1 && fits(a) && fits(a + 1)) {
            int differ = 0;
            for (int d = 0; d < 3; ++d) differ += cell[(int64_t)a * 3 + d] != cell[(int64_t)(a + 1) * 3 + d];
            pair = differ == 1;
        }
        if (pair) {
            paired[a] = 1;
            paired[a + 1] = 2;
            a += 2;
        } else {
            paired[a] = 0;
            a += 1;
        }
    }
}
struct PairCountIn {
    const uint8_t *paired;
    __device__ uint64_t operator()(int64_t a) const { return paired[a] == 1 ? 1u : 0u; }
};
// the big tiles of a box without the first run of a paired box
struct RestTileCountIn {
    const uint32_t *start;
    uint32_t ts;
    const uint8_t *paired;
    __device__ uint64_t operator()(int64_t a) const {
        const uint32_t cnt = start[a + 1] - start[a];
        return cnt / 64u + ((cnt & 63u) > ts ? 1u : 0u) - (paired[a] ? 1u : 0u);
    }
};

// flag[c] = 1 for every column c of a list (equal values from several threads: plain vector stores)
__global__ __launch_bounds__(256) void mark_cols_kernel(const uint32_t *__restrict__ cols, int64_t count,
                                                        uint32_t *__restrict__ flag) {
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (int64_t)gridDim.x * 256)
        flag[cols[e]] = 1u;
}

// work items counted per box by `count`: first[nb+1] (exclusive scan) and the box of every item
template <class CountIn>
static void build_items(CountIn count, int64_t nb, DevBuf<uint32_t> &first, DevBuf<uint32_t> &cbox, int64_t &nitems,
                        int64_t *tally, hipStream_t st) {
    first.alloc((size_t)nb + 1, tally);
    uint64_t total = 0;
    exclusive_scan(count, nb, U32Out{first.p}, &total, st);
    nitems = (int64_t)total;
    set_u32_kernel<<<1, 1, 0, st>>>(first.p + nb, (uint32_t)total);
    cbox.alloc((size_t)nitems, tally);
    if (nitems > 0)
        chunk_box_kernel<<<dim3((unsigned)cdiv(nitems, 256)), dim3(256), 0, st>>>(first.p, nb, nitems, cbox.p);
    F3M_HIP(hipGetLastError());
}

static void build_chunks(const uint32_t *start, int64_t nb, uint32_t chunk, DevBuf<uint32_t> &first,
                         DevBuf<uint32_t> &cbox, int64_t &nchunks, int64_t *tally, hipStream_t st,
                         const uint64_t *only_rows = nullptr, const uint32_t *only_flagged = nullptr) {
    first.alloc((size_t)nb + 1, tally);
    uint64_t total = 0;
    if (only_flagged)
        exclusive_scan(ChunkCountFlagIn{start, only_flagged, chunk}, nb, U32Out{first.p}, &total, st);
    else if (only_rows)
        exclusive_scan(ChunkCountIfIn{start, only_rows, chunk}, nb, U32Out{first.p}, &total, st);
    else
        exclusive_scan(ChunkCountIn{start, chunk}, nb, U32Out{first.p}, &total, st);
    nchunks = (int64_t)total;
    set_u32_kernel<<<1, 1, 0, st>>>(first.p + nb, (uint32_t)total);
    cbox.alloc((size_t)nchunks, tally);
    if (nchunks > 0)
        chunk_box_kernel<<<dim3((unsigned)cdiv(nchunks, 256)), dim3(256), 0, st>>>(first.p, nb, nchunks, cbox.p);
    F3M_HIP(hipGetLastError());
}

// ------------------------------------------------------------------------------------
// a point set while it is partitioned: the targets X of the plan, or the sources Y of a two-set plan
struct SetRef {
    const float *X;
    int64_t n;
    float *alpha;
    DevBuf<uint32_t> *keys, *perm;
    DevBuf<float> *Xs;
    f3m_level *lev;
};

// per-dimension minimum and the largest extent (one fp32 subtraction per dimension) of a set
template <int D>
static float set_bounds(const SetRef &S, const char *name, hipStream_t st) {
    DevBuf<float> part;
    DevBuf<int> bad;
    part.alloc((size_t)BBOX_BLOCKS * 2 * D);
    bad.alloc(1);
    F3M_HIP(hipMemsetAsync(bad.p, 0, sizeof(int), st));
    bbox_kernel<D><<<dim3(BBOX_BLOCKS), dim3(BBOX_NT), 0, st>>>(S.X, S.n, part.p, bad.p);
    F3M_HIP(hipGetLastError());
    std::vector<float> hp((size_t)BBOX_BLOCKS * 2 * D);
    int hbad = 0;
    F3M_HIP(hipMemcpyAsync(hp.data(), part.p, hp.size() * sizeof(float), hipMemcpyDeviceToHost, st));
    F3M_HIP(hipMemcpyAsync(&hbad, bad.p, sizeof(int), hipMemcpyDeviceToHost, st));
    F3M_HIP(hipStreamSynchronize(st));
    if (hbad) fail(F3M_ERR_NONFINITE, std::string(name) + " holds a NaN or an infinity");
    float E = 0.f;
    for (int d = 0; d < D; ++d) {
        float mn = INFINITY, mx = -INFINITY;
        for (int k = 0; k < BBOX_BLOCKS; ++k) {
            mn = std::min(mn, hp[(size_t)k * 2 * D + d]);
            mx = std::max(mx, hp[(size_t)k * 2 * D + D + d]);
        }
        volatile float ext = mx - mn;  // one fp32 subtraction
        if (ext > E) E = ext;
        S.alpha[d] = mn;
    }
    return E;
}

// Divide (Algorithm 1): the box table of depth l of one set -- heads of runs of equal depth-l keys,
// from the points or, once the boxes of the depth above are few against the points, from their
// intervals -- with parent ranks, child intervals of the depth above, cells and the largest box.
template <int D>
static void divide_set(f3m_plan_s &P, const SetRef &S, int l, DevBuf<uint32_t> &part, hipStream_t st) {
    int64_t *tally = &P.bytes;
    const int64_t n = S.n;
    f3m_level &lv = S.lev[l];
    const uint32_t *keys = S.keys->p;
    int shift = D * (P.Lq - l);
    const bool from_parents = l > 0 && (S.lev[l - 1].nb << D) <= n / 4;
    if (from_parents) {
        f3m_level &up = S.lev[l - 1];
        const int64_t nslots = up.nb << D;
        DevBuf<uint32_t> lb;
        lb.alloc((size_t)nslots + 1);
        child_bounds_kernel<D><<<dim3((unsigned)cdiv(nslots, 256)), dim3(256), 0, st>>>(keys, shift, up.start.p, nslots,
                                                                                      up.key.p, lb.p);
        F3M_HIP(hipGetLastError());
        set_u32_kernel<<<1, 1, 0, st>>>(lb.p + nslots, (uint32_t)n);
        ChildIn cin{lb.p};
        ScanState SS;
        scan_prepare(cin, nslots, SS, true, st);
        lv.nb = (int64_t)SS.total;
        lv.key.alloc((size_t)lv.nb, tally);
        lv.start.alloc((size_t)lv.nb + 1, tally);
        lv.parent.alloc((size_t)lv.nb, tally);
        up.cstart.alloc((size_t)up.nb + 1, tally);
        scan_finish(cin, nslots, SS, ChildOut<D>{lb.p, up.key.p, lv.start.p, lv.key.p, lv.parent.p, up.cstart.p}, st);
        set_u32_kernel<<<1, 1, 0, st>>>(lv.start.p + lv.nb, (uint32_t)n);
        set_u32_kernel<<<1, 1, 0, st>>>(up.cstart.p + up.nb, (uint32_t)lv.nb);
        F3M_HIP(hipStreamSynchronize(st));   // lb is released on leaving the scope
    } else {
        HeadIn hin{keys, shift};
        ScanState SS;
        scan_prepare(hin, n, SS, true, st);
        lv.nb = (int64_t)SS.total;
        lv.key.alloc((size_t)lv.nb, tally);
        lv.start.alloc((size_t)lv.nb + 1, tally);
        scan_finish(hin, n, SS, HeadOut{keys, shift, lv.start.p, lv.key.p}, st);
        set_u32_kernel<<<1, 1, 0, st>>>(lv.start.p + lv.nb, (uint32_t)n);
    }
    {
        int grid = (int)std::min<int64_t>(1024, cdiv(lv.nb, 256));
        max_count_kernel<<<dim3(grid), dim3(256), 0, st>>>(lv.start.p, lv.nb, part.p);
        F3M_HIP(hipGetLastError());
        std::vector<uint32_t> hp(grid);
        F3M_HIP(hipMemcpyAsync(hp.data(), part.p, grid * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        F3M_HIP(hipStreamSynchronize(st));
        lv.max_box = *std::max_element(hp.begin(), hp.end());
    }
    lv.cell.alloc((size_t)lv.nb * D, tally);
    cells_kernel<D><<<dim3((unsigned)cdiv(lv.nb, 256)), dim3(256), 0, st>>>(lv.key.p, lv.nb, l, lv.cell.p);
    F3M_HIP(hipGetLastError());
    if (from_parents) {
        // parent ranks and child intervals came with the division
    } else if (l > 0) {
        lv.parent.alloc((size_t)lv.nb, tally);
        f3m_level &up = S.lev[l - 1];
        up.cstart.alloc((size_t)up.nb + 1, tally);
        HeadIn pin{lv.key.p, D};
        uint64_t tot = 0;
        exclusive_scan(pin, lv.nb, ParentOut{lv.parent.p, up.cstart.p}, &tot, st);
        if ((int64_t)tot != up.nb) fail(F3M_ERR_HIP, "internal: parent count mismatch");
        set_u32_kernel<<<1, 1, 0, st>>>(up.cstart.p + up.nb, (uint32_t)lv.nb);
    } else {
        lv.parent.alloc((size_t)lv.nb, tally);
        F3M_HIP(hipMemsetAsync(lv.parent.p, 0, sizeof(uint32_t), st));
    }
}

template <int D>
static void build_plan_d(f3m_plan_s &P, const float *X, const float *Y, hipStream_t st) {
    const int64_t n = P.n;
    int64_t *tally = &P.bytes;
    for (int k = 0; k < 8; ++k) F3M_HIP(hipEventCreate(&P.ev[k]));
    F3M_HIP(hipEventRecord(P.ev[0], st));
    // the set(s) to partition: the targets, and the sources when they are another set
    std::vector<SetRef> sets;
    sets.push_back(SetRef{X, n, P.alpha, &P.keys, &P.perm, &P.Xs, P.lev});
    if (P.src) sets.push_back(SetRef{Y, P.src->n, P.src->alpha, &P.src->keys, &P.src->perm, &P.src->Xs, P.src->lev});

    // ---- enclosing cubes: a common edge, the largest extent of either set (Sec. 3), each set
    //      anchored at its own per-dimension minimum (the alpha of the box-index formula, Sec. 4.2)
    {
        float E = 0.f;
        for (size_t k = 0; k < sets.size(); ++k) E = std::max(E, set_bounds<D>(sets[k], k ? "Y" : "X", st));
        P.E = E;
        P.scale = E > 0.f ? (float)(std::ldexp(1.0, P.Lq) / (double)E) : 0.f;
    }

    // ---- keys, sort, gather
    for (const SetRef &S : sets) {
        // (one tile of slack behind the keys and the indices: the sort reads whole tiles)
        S.keys->alloc((size_t)S.n + RS_TILE, tally);
        S.perm->alloc((size_t)S.n + RS_TILE, tally);
        AlphaArg aa;
        for (int d = 0; d < F3M_MAX_DIM; ++d) aa.a[d] = S.alpha[d];
        keys_kernel<D><<<dim3((unsigned)cdiv(S.n, 256)), dim3(256), 0, st>>>(S.X, S.n, aa, P.scale, P.Lq, S.keys->p);
        F3M_HIP(hipGetLastError());
    }
    F3M_HIP(hipEventRecord(P.ev[1], st));
    int bits_sorted = 0;
    for (const SetRef &S : sets) {
        DevBuf<uint32_t> keys_b, perm_b;
        keys_b.alloc((size_t)S.n + RS_TILE);
        perm_b.alloc((size_t)S.n + RS_TILE);
        int bits = P.E > 0.f ? D * P.Lq : 0;
        bits_sorted = bits;
        bool in_b;
        if (bits == 0) {
            iota_kernel<<<dim3((unsigned)cdiv(S.n, 256)), dim3(256), 0, st>>>(S.perm->p, S.n);
            in_b = false;
        } else {
            in_b = radix_sort(S.keys->p, S.perm->p, keys_b.p, perm_b.p, S.n, bits, st);
        }
        if (in_b) {
            std::swap(S.keys->p, keys_b.p);
            std::swap(S.perm->p, perm_b.p);
        }
        F3M_HIP(hipStreamSynchronize(st));   // the second buffers are released on leaving the scope
    }
    F3M_HIP(hipEventRecord(P.ev[2], st));
    for (size_t k = 0; k < sets.size(); ++k) {
        const SetRef &S = sets[k];
        // 64 zero points of padding after the last point: kernels may read whole 32-point blocks
        S.Xs->alloc(((size_t)S.n + PAD_POINTS) * D, tally);
        F3M_HIP(hipMemsetAsync(S.Xs->p + (size_t)S.n * D, 0, (size_t)PAD_POINTS * D * sizeof(float), st));
        // A large set goes through the three-pass permutation, whose tables also serve every product
        // (route.hip); its points follow the same way when they have three coordinates.
        std::unique_ptr<f3m_route> &route = k ? P.src->route : P.route;
        if (S.n >= P.route_min_n && bits_sorted > 0) {
            route.reset(new f3m_route());
            route_build(*route, S.perm->p, S.n, tally, st);
        }
        if (route && D == 3) {
            DevBuf<float> tmp;
            tmp.alloc((size_t)S.n * 3);
            route_gather_rows3(*route, S.X, S.Xs->p, tmp.p, st);
            F3M_HIP(hipStreamSynchronize(st));   // `tmp` is released on leaving the scope
        } else {
            gather_rows_kernel<D><<<dim3((unsigned)cdiv(S.n, 256)), dim3(256), 0, st>>>(S.X, S.perm->p, S.n, S.Xs->p);
            F3M_HIP(hipGetLastError());
        }
    }
    F3M_HIP(hipEventRecord(P.ev[3], st));
    F3M_HIP(hipStreamSynchronize(st));

    // ---- Algorithm 1 loop: divide, new interactions, partition
    int cap = P.Lq;
    if (P.max_depth > 0 && P.max_depth < cap) cap = P.max_depth;
    if (cap > F3M_MAX_LEVELS) cap = F3M_MAX_LEVELS;
    if (!(P.E > 0.f)) cap = 0;
    DevBuf<uint32_t> part;
    part.alloc(1024);
    float t_boxes = 0.f, t_lists = 0.f;
    hipEvent_t ea = P.ev[4], eb = P.ev[5], ec = P.ev[6];
    int l = 0;
    for (;; ++l) {
        f3m_level &lv = P.lev[l];
        F3M_HIP(hipEventRecord(ea, st));
        for (const SetRef &S : sets) divide_set<D>(P, S, l, part, st);
        const f3m_level &sv = P.slev(l);
        F3M_HIP(hipEventRecord(eb, st));

        // new interactions + partition
        lv.near_ptr.alloc((size_t)lv.nb + 1, tally);
        lv.far_ptr.alloc((size_t)lv.nb + 1, tally);
        if (l == 0) {
            lv.near_col.alloc(1, tally);
            lv.far_col.alloc(1, tally);
            F3M_HIP(hipMemsetAsync(lv.near_ptr.p, 0, 2 * sizeof(uint64_t), st));
            F3M_HIP(hipMemsetAsync(lv.far_ptr.p, 0, 2 * sizeof(uint64_t), st));
            F3M_HIP(hipMemsetAsync(lv.near_col.p, 0, sizeof(uint32_t), st));
            set_u64_kernel<<<1, 1, 0, st>>>(lv.near_ptr.p + 1, 1ull);
            lv.near_sz = 1;
            lv.far_sz = 0;
        } else {
            f3m_level &up = P.lev[l - 1];
            const f3m_level &sup = P.slev(l - 1);
            DevBuf<uint32_t> cn, cf, cs;
            cn.alloc((size_t)lv.nb);
            cf.alloc((size_t)lv.nb);
            if (P.rho > 0) cs.alloc((size_t)lv.nb);
            unsigned grid = (unsigned)cdiv(lv.nb, 128);
            // Sec. 4.3: once the boxes pass the smoothness criterion every pair left is interpolated
            lv.smooth = !P.force_all_near && smooth_rule((double)P.E, l, D, (double)P.gamma, (double)P.eta_smooth);
            if (lv.smooth) P.smooth_depth = l;
            ListArg A = list_rules(P, l);
            A.cnt_near = cn.p;
            A.cnt_far = cf.p;
            A.cnt_small = cs.p;
            if constexpr (D <= 3) {
                if (lists_by_parent(A, D))
                    lists_parent_kernel<D><<<dim3((unsigned)((up.nb + 7) / 8 * 8)), dim3(64), 0, st>>>(0, up.nb, up.cstart.p, lv.cell.p,
                                                                                       up.near_ptr.p, up.near_col.p, A);
                else
                    lists_kernel<D><<<dim3(grid), dim3(128), 0, st>>>(0, lv.nb, lv.parent.p, lv.cell.p, up.near_ptr.p,
                                                                     up.near_col.p, sup.cstart.p, A);
            } else {
                lists_kernel<D><<<dim3(grid), dim3(128), 0, st>>>(0, lv.nb, lv.parent.p, lv.cell.p, up.near_ptr.p,
                                                                 up.near_col.p, sup.cstart.p, A);
            }
            F3M_HIP(hipGetLastError());
            uint64_t tn = 0, tf = 0, ts = 0;
            exclusive_scan(U32In{cn.p}, lv.nb, PtrOut{lv.near_ptr.p}, &tn, st);
            exclusive_scan(U32In{cf.p}, lv.nb, PtrOut{lv.far_ptr.p}, &tf, st);
            set_u64_kernel<<<1, 1, 0, st>>>(lv.near_ptr.p + lv.nb, tn);
            set_u64_kernel<<<1, 1, 0, st>>>(lv.far_ptr.p + lv.nb, tf);
            if (P.rho > 0) {
                lv.small_ptr.alloc((size_t)lv.nb + 1, tally);
                exclusive_scan(U32In{cs.p}, lv.nb, PtrOut{lv.small_ptr.p}, &ts, st);
                set_u64_kernel<<<1, 1, 0, st>>>(lv.small_ptr.p + lv.nb, ts);
                lv.small_col.alloc((size_t)ts, tally);
            }
            lv.near_sz = (int64_t)tn;
            lv.far_sz = (int64_t)tf;
            lv.small_sz = (int64_t)ts;
            lv.near_col.alloc((size_t)tn, tally);
            lv.p = P.adaptive_far ? adaptive_nodes((double)P.E, l, (double)P.gamma, P.p) : P.p;
            lv.r = 1;
            for (int d = 0; d < D; ++d) lv.r *= lv.p;
            if (tf > 0 && m2l_stencil_applies(P) && (lv.p == 4 || lv.p == 0)) {
                // the M2L of this depth enumerates the far partners itself (candidate grid around the
                // parent): only the row lengths are kept
                lv.far_implicit = true;
                lv.far_col.alloc(0, tally);
            } else {
                lv.far_col.alloc((size_t)tf, tally);
            }
            A.near_ptr = lv.near_ptr.p;
            A.far_ptr = lv.far_ptr.p;
            A.small_ptr = lv.small_ptr.p;
            A.near_col = lv.near_col.p;
            A.far_col = lv.far_implicit ? nullptr : lv.far_col.p;
            A.small_col = lv.small_col.p;
            if constexpr (D == 3) {
                // the tables of the candidate-grid M2L come out of the same enumeration
                if (lists_by_parent(A, D) && lv.far_implicit && lv.p != 0 && stencil_tables_alloc(P, l, st)) {
                    A.st_cand = lv.st_cand.p;
                    A.st_child = lv.st_child.p;
                }
            }
            if constexpr (D <= 3) {
                if (lists_by_parent(A, D))
                    lists_parent_kernel<D><<<dim3((unsigned)((up.nb + 7) / 8 * 8)), dim3(64), 0, st>>>(1, up.nb, up.cstart.p, lv.cell.p,
                                                                                       up.near_ptr.p, up.near_col.p, A);
                else
                    lists_kernel<D><<<dim3(grid), dim3(128), 0, st>>>(1, lv.nb, lv.parent.p, lv.cell.p, up.near_ptr.p,
                                                                     up.near_col.p, sup.cstart.p, A);
            } else {
                lists_kernel<D><<<dim3(grid), dim3(128), 0, st>>>(1, lv.nb, lv.parent.p, lv.cell.p, up.near_ptr.p,
                                                                 up.near_col.p, sup.cstart.p, A);
            }
            F3M_HIP(hipGetLastError());
            F3M_HIP(hipStreamSynchronize(st));
        }
        F3M_HIP(hipEventRecord(ec, st));
        F3M_HIP(hipStreamSynchronize(st));
        float ms = 0.f;
        F3M_HIP(hipEventElapsedTime(&ms, ea, eb));
        t_boxes += ms;
        F3M_HIP(hipEventElapsedTime(&ms, eb, ec));
        t_lists += ms;
        // while interactions remain and the largest box of either tree is above zeta (Algorithm 1)
        if (!(lv.near_sz > 0 && lv.max_box > P.leaf_max && sv.max_box > P.leaf_max && l < cap)) break;
    }
    P.L = l;

    // ---- work splits and workspaces
    F3M_HIP(hipEventRecord(ea, st));
    // With D = 3 and 4 nodes per dimension node weights and node potentials are passed between
    // depths, so only the last depth streams the points.
    // the band of depths with implicit far rows and 4 nodes per dimension (under the adaptive rule
    // the deepest depths may use 3 nodes and the coarsest may be dropped)
    // (with 4 nodes per dimension in 3-D; the M2L of a depth in the band is the candidate-grid one where
    // that applies, else the one that works from the far list: two point sets, other far ratios)
    auto in_band = [&](int k) { return D == 3 && k >= 2 && P.lev[k].far_sz > 0 && P.lev[k].p == 4; };
    for (int k = P.L; k >= 2 && P.tree_lmax == 0; --k)
        if (in_band(k)) P.tree_lmax = k;
    if (P.tree_lmax > 0) {
        P.tree_lmin = P.tree_lmax;
        while (in_band(P.tree_lmin - 1)) --P.tree_lmin;
        upload_transfer(P, st);
    }
    upload_kron_tables(P, st);
    build_far_orders(P, st);
    for (int k = 1; k <= P.L; ++k) build_stencil_tables(P, k, st);
    int64_t max_w = 0, max_v = 0, max_part = 0, max_slice = 0;
    for (int k = 1; k <= P.L; ++k) {
        f3m_level &lv = P.lev[k];
        if (lv.far_sz == 0 || lv.p == 0) continue;   // nothing to interpolate, or dropped
        const bool tree = P.tree_lmin > 0 && k >= P.tree_lmin && k <= P.tree_lmax;
        f3m_level &sv = P.slev(k);
        if (tree) {
            // Node potentials are passed down the targets' tree.  One point set: node weights are passed up
            // the same tree, and carry one row of zeros behind the last box (what the candidate-grid M2L reads
            // for an absent candidate).  Two point sets: the node weights of every depth come from the points.
            lv.Vl.alloc((size_t)lv.nb * lv.r, tally);
            if (!P.src) {
                lv.Wl.alloc((size_t)(lv.nb + 1) * lv.r, tally);
                F3M_HIP(hipMemsetAsync(lv.Wl.p + (size_t)lv.nb * lv.r, 0, (size_t)lv.r * sizeof(float), st));
                if (k < P.tree_lmax) continue;   // only the last depth of the band needs chunks
            }
        }
        // runs of points for the L2P (targets: in the band only its last depth) and the P2M (sources: the
        // same runs for one point set)
        if (!tree || k == P.tree_lmax)
            build_chunks(lv.start.p, lv.nb, P2M_CHUNK, lv.chunk_first, lv.chunk_box, lv.nchunks, tally, st);
        if (P.src) {
            // Only the source boxes that occur in a far row of this depth need node weights (the two sets
            // may overlap in a small part of the sources' cube only).
            DevBuf<uint32_t> used;
            used.alloc((size_t)sv.nb);
            F3M_HIP(hipMemsetAsync(used.p, 0, (size_t)sv.nb * sizeof(uint32_t), st));
            mark_cols_kernel<<<dim3((unsigned)std::min<int64_t>(cdiv(lv.far_sz, 256), 1 << 20)), dim3(256), 0, st>>>(
                lv.far_col.p, lv.far_sz, used.p);
            F3M_HIP(hipGetLastError());
            build_chunks(sv.start.p, sv.nb, P2M_CHUNK, sv.chunk_first, sv.chunk_box, sv.nchunks, tally, st, nullptr,
                         used.p);
            F3M_HIP(hipStreamSynchronize(st));   // `used` is released on leaving the scope
        }
        if (sv.max_box > (int64_t)P2M_CHUNK * P2M_SLICE * 2) {
            // a box with more than a thousand chunks: its partial node weights are summed in two stages
            build_chunks(sv.chunk_first.p, sv.nb, P2M_SLICE, sv.slice_first, sv.slice_box, sv.nslices, tally, st);
            max_slice = std::max(max_slice, sv.nslices * (int64_t)lv.r);
        }
        if (!tree || P.src) max_w = std::max(max_w, sv.nb * (int64_t)lv.r);
        if (!tree) max_v = std::max(max_v, lv.nb * (int64_t)lv.r);
        max_part = std::max(max_part, sv.nchunks * (int64_t)lv.r);
    }
    {
        const f3m_level &lf = P.lev[P.L];
        // Few boxes: rows are long, and the near field splits every tile over several wavefronts; an overflow
        // tile would leave its whole row to one wavefront, so there are none (every run is a tile of its own).
        const uint32_t ts = lf.nb < 8192 ? 0u : (uint32_t)overflow_targets(D);
        build_items(BigTileCountIn{lf.start.p, ts}, lf.nb, P.tile_first, P.tile_box, P.ntiles, tally, st);
        build_items(OverflowTileCountIn{lf.start.p, ts}, lf.nb, P.otile_first, P.otile_box, P.notiles, tally, st);
        // tiles worked in pairs (the rows must come from the plain far rule: the kernel tells the shared near
        // boxes of a pair by it)
        if (P.L >= 1 && ts > 0 && lf.near_sz > 0 && !lf.smooth && P.rho == 0 && p2p_pairs_allowed(P)) {
            const f3m_level &up = P.lev[P.L - 1];
            P.paired.alloc((size_t)lf.nb, tally);
            pair_flag_kernel<<<dim3((unsigned)cdiv(up.nb, 256)), dim3(256), 0, st>>>(
                up.nb, up.cstart.p, lf.cell.p, lf.start.p, lf.near_ptr.p, ts, P.paired.p);
            F3M_HIP(hipGetLastError());
            build_items(PairCountIn{P.paired.p}, lf.nb, P.pair_first, P.pair_box, P.npairs, tally, st);
            build_items(RestTileCountIn{lf.start.p, ts, P.paired.p}, lf.nb, P.rtile_first, P.rtile_box, P.nrtiles, tally, st);
        }
    }
    // target tiles of the small-field rows of every depth (Sec. 4.2)
    for (int k = 1; k <= P.L; ++k) {
        f3m_level &lv = P.lev[k];
        if (lv.small_sz > 0)
            build_chunks(lv.start.p, lv.nb, D <= 4 ? 16 : 8, lv.sm_tile_first, lv.sm_tile_box, lv.sm_ntiles, tally, st,
                         lv.small_ptr.p);   // runs of targets as p2p_small_kernel takes them
    }
    {
        // partial sums of a near field whose tiles are split over several wavefronts (few targets, long rows)
        const int nsplit = P.lev[P.L].near_sz > 0 ? p2p_nsplit(P, P.L, P.ntiles) : 1;
        if (nsplit > 1) P.p2p_part.alloc((size_t)nsplit * (size_t)n, tally);
    }
    if (P.route || (P.src && P.src->route)) {
        const size_t m = (size_t)std::max<int64_t>(P.route ? n : 0, (P.src && P.src->route) ? P.src->n : (P.route ? n : 0));
        P.route_a.alloc(m, tally);
        P.route_b.alloc(m, tally);
    }
    P.bs.alloc((size_t)P.ns() + PAD_POINTS, tally);
    F3M_HIP(hipMemsetAsync(P.bs.p + P.ns(), 0, (size_t)PAD_POINTS * sizeof(float), st));
    P.ys.alloc((size_t)n, tally);
    P.yn.alloc((size_t)n, tally);
    if (!P.no_overlap) F3M_HIP(hipStreamCreateWithFlags(&P.side, hipStreamNonBlocking));
    for (hipEvent_t *e : {&P.ev_fork, &P.ev_join, &P.ev_p2p0, &P.ev_p2p1}) F3M_HIP(hipEventCreate(e));
    P.W.alloc((size_t)max_w, tally);
    P.V.alloc((size_t)max_v, tally);
    P.Wpart.alloc((size_t)max_part, tally);
    P.Wslice.alloc((size_t)max_slice, tally);
    F3M_HIP(hipEventRecord(eb, st));
    F3M_HIP(hipStreamSynchronize(st));

    float ms = 0.f;
    F3M_HIP(hipEventElapsedTime(&P.times.bbox_keys, P.ev[0], P.ev[1]));
    F3M_HIP(hipEventElapsedTime(&P.times.sort, P.ev[1], P.ev[2]));
    F3M_HIP(hipEventElapsedTime(&P.times.gather, P.ev[2], P.ev[3]));
    P.times.boxes = t_boxes;
    P.times.lists = t_lists;
    F3M_HIP(hipEventElapsedTime(&P.times.tables, ea, eb));
    F3M_HIP(hipEventElapsedTime(&ms, P.ev[0], eb));
    P.times.plan_total = ms;
    P.have_plan_times = true;
}

// Far rows (CSR columns, ascending) of a depth that keeps only their lengths: the fill pass of
// the list kernel with the near side switched off.  cols_dev holds far_sz entries.
void materialize_far(const f3m_plan_s &P, int level, uint32_t *cols_dev, hipStream_t st) {
    const f3m_level &lv = P.lev[level], &up = P.lev[level - 1];
    const unsigned grid = (unsigned)cdiv(lv.nb, 128);
    ListArg A = list_rules(P, level);
    A.far_ptr = lv.far_ptr.p;
    A.far_col = cols_dev;
    auto launch = [&](auto kern) {
        kern<<<dim3(grid), dim3(128), 0, st>>>(1, lv.nb, lv.parent.p, lv.cell.p, up.near_ptr.p, up.near_col.p,
                                               P.slev(level - 1).cstart.p, A);
    };
    switch (P.D) {
        case 1: launch(lists_kernel<1>); break;
        case 2: launch(lists_kernel<2>); break;
        case 3: launch(lists_kernel<3>); break;
        case 4: launch(lists_kernel<4>); break;
        case 5: launch(lists_kernel<5>); break;
        case 6: launch(lists_kernel<6>); break;
        default: launch(lists_kernel<7>); break;
    }
    F3M_HIP(hipGetLastError());
    F3M_HIP(hipStreamSynchronize(st));
}

// Point pairs behind the near list of the last depth and the far lists of every depth (for
// reports and the coverage identity near + far = n^2); computed on first request because it
// re-reads every list.
void compute_far_point_pairs(f3m_plan_s &P) {
    if (P.have_far_point_pairs) return;
    {
        ScanState S;
        const f3m_level &lf = P.lev[P.L];
        scan_prepare(NearPairsIn{lf.start.p, P.slev(P.L).start.p, lf.near_ptr.p, lf.near_col.p}, lf.nb, S, true, nullptr);
        P.near_point_pairs = (int64_t)S.total;
    }
    for (int l = 1; l <= P.L; ++l) {
        f3m_level &lv = P.lev[l];
        lv.small_point_pairs = 0;
        if (lv.small_sz > 0) {
            ScanState S;
            scan_prepare(NearPairsIn{lv.start.p, P.slev(l).start.p, lv.small_ptr.p, lv.small_col.p}, lv.nb, S, true, nullptr);
            lv.small_point_pairs = (int64_t)S.total;
        }
        lv.far_point_pairs = 0;
        if (lv.far_sz == 0) continue;
        if (lv.far_implicit) {
            DevBuf<uint32_t> cols;
            cols.alloc((size_t)lv.far_sz);
            materialize_far(P, l, cols.p, nullptr);
            ScanState S;
            scan_prepare(NearPairsIn{lv.start.p, P.slev(l).start.p, lv.far_ptr.p, cols.p}, lv.nb, S, true, nullptr);
            lv.far_point_pairs = (int64_t)S.total;
        } else {
            ScanState S;
            scan_prepare(NearPairsIn{lv.start.p, P.slev(l).start.p, lv.far_ptr.p, lv.far_col.p}, lv.nb, S, true, nullptr);
            lv.far_point_pairs = (int64_t)S.total;
        }
    }
    P.have_far_point_pairs = true;
}

// Smoothness criterion with the O(1) bound of Sec. 4.3: a box of edge l has an effective variance
// of at most D l^2 / (8 gamma^2), two boxes D l^2 / (4 gamma^2); adjacent pairs are interpolated
// when that is <= eta_smooth.
bool smooth_rule(double E, int depth, int D, double gamma, double eta_smooth) {
    if (!(eta_smooth > 0.0)) return false;
    const double l = E / std::ldexp(1.0, depth);
    return (double)D * l * l / (4.0 * gamma * gamma) <= eta_smooth;
}

// Adaptive far-field rule of Sec. 4.3 on q = l^2 / (2 gamma^2): min(p, 3) nodes per dimension if
// q <= 0.01 (the paper's min(r, 3^D) on a tensor grid), p if q <= 5, 0 (dropped) above.
int adaptive_nodes(double E, int depth, double gamma, int p) {
    const double l = E / std::ldexp(1.0, depth);
    const double q = l * l / (2.0 * gamma * gamma);
    if (q <= 0.01) return p < 3 ? p : 3;
    if (q <= 5.0) return p;
    return 0;
}

void build_plan(f3m_plan_s &P, const float *X, const float *Y, hipStream_t st) {
    switch (P.D) {
        case 1: build_plan_d<1>(P, X, Y, st); break;
        case 2: build_plan_d<2>(P, X, Y, st); break;
        case 3: build_plan_d<3>(P, X, Y, st); break;
        case 4: build_plan_d<4>(P, X, Y, st); break;
        case 5: build_plan_d<5>(P, X, Y, st); break;
        case 6: build_plan_d<6>(P, X, Y, st); break;
        case 7: build_plan_d<7>(P, X, Y, st); break;
        default: fail(F3M_ERR_INVALID_ARG, "D must be in [1,7]");
    }
}

}  // namespace f3m
