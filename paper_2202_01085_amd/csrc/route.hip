// Permutations of 1e8 .. 2e9 values between the caller's point order and the plan's box order (the
// reindexing vector sigma of Sec. 4.2; grouping of Sec. 4.1) as three streaming passes through LDS.
//
// A plain gather b[perm[k]] (or scatter) of a random permutation touches one 128-byte line per 4-byte value
// once the array is larger than the caches: 130 GB of traffic for 4 GB at n = 1e9.  Here a value travels
//     box order k  --pass 1-->  order p1  --pass 2-->  order p2  --pass 3-->  caller's order i = perm[k]
// where, with windows of T = 32768 consecutive caller indices (w = i >> 15, split as w = d1 * B2 + d2):
//   pass 1  deals every tile of T consecutive k into B1 <= 256 buckets by d1 (bucket d1 holds exactly the
//           2^15 B2 values whose destination lies in its B2 windows, so it starts at d1 2^15 B2);
//   pass 2  deals every tile of T consecutive p1 (a tile lies inside one bucket) into the B2 windows of that
//           bucket (window w receives exactly its T values, at w T ...);
//   pass 3  puts the T values of a window in their places inside LDS and writes the window out in one piece.
// (T = 32768 because 128 KB of the 160 KB of LDS then hold one tile of floats.)
// Every pass reads and writes runs that are contiguous in memory (some hundred values per bucket and tile),
// and the places (the position of a value in the LDS copy of its tile, 16 bits per value and pass) depend on
// perm only: they are computed once per plan by route_build, so a pass moves data and does nothing else.
// The gather direction (caller's order -> box order) runs the same three passes backwards with the same tables.
#include "plan.h"

namespace f3m {

constexpr int RT_BITS = 15;
constexpr int RT_TILE = 1 << RT_BITS;    // values per tile and per window
constexpr int RT_NT = 1024;              // threads of a workgroup: one tile
constexpr int RT_IPT = RT_TILE / RT_NT;  // 32 values per thread
constexpr int RT_NW = RT_NT / 64;        // 16 wavefronts

struct RouteLevel {
    int shift;        // digit of a destination index: (i >> shift) & mask
    uint32_t mask;
    int second;       // 0: pass 1 (buckets over all tiles), 1: pass 2 (windows inside the bucket of the tile)
    int s2;           // B2 = 1 << s2 tiles per bucket of pass 1
    int B;            // digits of this pass
    int64_t ntiles;
};

// Tile of this workgroup.  Workgroups go to the 8 dies (each with its own L2) in turn; every die takes a
// contiguous range of tiles, so that the runs which neighbouring tiles write to (or read from) the same bucket
// meet in one L2 as whole lines.  The grid holds a whole number of rounds over the dies (route_grid); a
// workgroup beyond the last tile returns at once.
__device__ inline int64_t route_tile(int64_t n) {
    const int64_t ntiles = (n + RT_TILE - 1) / RT_TILE, per_die = (ntiles + 7) >> 3;
    const int64_t t = (int64_t)(blockIdx.x & 7u) * per_die + (int64_t)(blockIdx.x >> 3);
    return t < ntiles ? t : -1;
}
static unsigned route_grid(int64_t ntiles) { return (unsigned)((ntiles + 7) / 8 * 8); }

// Where the runs of a pass begin.  The buckets of pass 1 and the windows of pass 2 have known sizes (bucket d1
// holds exactly the values bound for its B2 windows, a window its T values), so their first positions need no
// counting: bucket d1 starts at d1 B2 T, window w at w T.  A tile reserves the run of each of its digits by an
// atomic add on the cursor of the bucket (pass 1) or window (pass 2); the order of the runs inside a bucket is
// then the order in which the tiles got there, which is as good as any: the places of the later passes are
// computed from the order that came out, and the values end where perm says whatever the order in between.
__global__ __launch_bounds__(256) void route_cursor_init_kernel(uint32_t *__restrict__ cursor, int64_t count,
                                                                uint32_t step) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) cursor[i] = (uint32_t)i * step;
}

// One tile of a pass: the place of every value in the LDS copy of the tile (values of a digit together,
// digits ascending, inside a digit in tile order), the destinations moved along to the next order, and the
// tile's tables (first place of each digit; global position of the tile's first value of each digit, minus
// that place).  Tile order = (wavefront, round, lane); ranking against per-wave LDS counters.
__global__ __launch_bounds__(RT_NT) void route_rank_kernel(const uint32_t *__restrict__ dest_in, int64_t n, RouteLevel R,
                                                           uint32_t *__restrict__ cursor,
                                                           uint16_t *__restrict__ slot, uint32_t *__restrict__ dest_out,
                                                           uint16_t *__restrict__ off_out,
                                                           uint32_t *__restrict__ dstart_out,
                                                           uint32_t *__restrict__ gofs_out) {
    const int64_t tb = route_tile(n);
    if (tb < 0) return;
    __shared__ uint32_t wcnt[RT_NW][256];   // per wave: values of each digit seen so far; later the wave's offset
    __shared__ uint32_t dstart[257];        // first place of each digit
    __shared__ uint32_t gbase[256];         // global position of the tile's first value of each digit
    __shared__ __attribute__((aligned(8))) uint32_t skey[RT_TILE];
    // per wave, while the values are ranked (skey is not in use yet): the lanes that hold each digit in the current round
    uint64_t (*wmask)[256] = reinterpret_cast<uint64_t (*)[256]>(skey);
    static_assert(sizeof(uint64_t) * RT_NW * 256 <= sizeof(uint32_t) * RT_TILE, "the lane masks must fit the tile buffer");
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid < 256) {
#pragma unroll
        for (int k = 0; k < RT_NW; ++k) {
            wcnt[k][tid] = 0;
            wmask[k][tid] = 0ull;
        }
    }
    __syncthreads();
    const uint64_t mybit = 1ull << lane;
    const int64_t tile0 = tb * RT_TILE;
    const int64_t base = tile0 + (int64_t)w * (RT_IPT * 64);
    uint32_t rk[RT_IPT / 2];   // rank within (wave, digit), below 2048: two per register
#pragma unroll
    for (int r = 0; r < RT_IPT / 2; ++r) rk[r] = 0u;
#pragma unroll
    for (int h = 0; h < RT_IPT; h += 8) {   // eight rounds at a time: their loads are in flight together
        uint32_t key[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int64_t i = base + (h + r) * 64 + lane;
            key[r] = i < n ? dest_in[i] : 0u;
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int64_t i = base + (h + r) * 64 + lane;
            const bool valid = i < n;
            const uint32_t digit = (key[r] >> R.shift) & R.mask;
            // The lanes of the round with the same digit find each other through LDS: every lane ORs its own
            // bit into the 64-bit word of its digit (an atomic OR: the result does not depend on the order),
            // reads the word back and counts the bits below its own; the first lane of each group adds the
            // group to the digit's running count and clears the word.  (The wave runs in lockstep and its
            // LDS operations complete in order.)
            if (valid) {
                atomicOr(reinterpret_cast<unsigned long long *>(&wmask[w][digit]), (unsigned long long)mybit);
                __builtin_amdgcn_wave_barrier();
                const uint64_t peers = wmask[w][digit];
                const uint32_t cnt = wcnt[w][digit];
                const uint32_t before =
                    __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u));
                rk[(h + r) / 2] |= (cnt + before) << (16 * ((h + r) & 1));
                __builtin_amdgcn_wave_barrier();
                if (before == 0) {
                    wcnt[w][digit] = cnt + (uint32_t)__popcll(peers);
                    wmask[w][digit] = 0ull;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    // per digit: the waves' counts become the waves' offsets; the totals go to dstart
    if (tid < 256) {
        uint32_t run = 0;
#pragma unroll
        for (int k = 0; k < RT_NW; ++k) {
            const uint32_t c = wcnt[k][tid];
            wcnt[k][tid] = run;
            run += c;
        }
        dstart[tid] = run;
    }
    __syncthreads();
    if (w == 0) {   // exclusive prefix sum of the 256 totals: four digits per lane
        uint32_t v[4], s = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[k] = dstart[lane * 4 + k]; s += v[k]; }
        uint32_t ex = wave_incl_scan_u32(s) - s;
#pragma unroll
        for (int k = 0; k < 4; ++k) { dstart[lane * 4 + k] = ex; ex += v[k]; }
        if (lane == 63) dstart[256] = ex;
    }
    __syncthreads();
    // the runs of this tile: digit b takes the next dstart[b + 1] - dstart[b] positions of its bucket (pass 1)
    // or of its window inside the bucket of this tile (pass 2)
    if (tid < 256) {
        uint32_t g = 0;
        if (tid < R.B) {
            const uint32_t count = dstart[tid + 1] - dstart[tid];
            const int64_t c = R.second ? ((tb >> R.s2) << R.s2) + tid : (int64_t)tid;
            if (count > 0) g = atomicAdd(&cursor[c], count);
        }
        gbase[tid] = g;
    }
#pragma unroll
    for (int h = 0; h < RT_IPT; h += 8) {
        uint32_t key[8];   // read again: keeping the first copy would not fit the registers
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int64_t i = base + (h + r) * 64 + lane;
            key[r] = i < n ? dest_in[i] : 0u;
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int64_t i = base + (h + r) * 64 + lane;
            if (i < n) {
                const uint32_t digit = (key[r] >> R.shift) & R.mask;
                const uint32_t pos = dstart[digit] + wcnt[w][digit] + ((rk[(h + r) / 2] >> (16 * ((h + r) & 1))) & 0xFFFFu);
                skey[pos] = key[r];
                slot[i] = (uint16_t)pos;
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // keeps the chunks apart: all 32 loads at once would not fit the registers
    }
    __syncthreads();
    const int64_t left = n - tile0;
    const int cntile = (int)(left < RT_TILE ? left : RT_TILE);
#pragma unroll 4
    for (int r = 0; r < RT_IPT; ++r) {
        const int pos = r * RT_NT + tid;
        if (pos < cntile) {
            const uint32_t k = skey[pos];
            const uint32_t digit = (k >> R.shift) & R.mask;
            const uint32_t g = gbase[digit] + ((uint32_t)pos - dstart[digit]);
            // the last pass needs no more than the place inside the window
            if (off_out) off_out[g] = (uint16_t)(k & (RT_TILE - 1));
            else dest_out[g] = k;
        }
    }
    if (tid <= 256) dstart_out[tb * 257 + tid] = dstart[tid];
    if (tid < 256) gofs_out[tb * 256 + tid] = gbase[tid] - dstart[tid];
}

// ------------------------------------------------------------------------------------
// the passes.  A source or destination with several components per value (the rows of X) is addressed as
// base[(index) * stride + component]; the orders between the passes hold one array per component.
// ------------------------------------------------------------------------------------
// digit whose run of places [ds[b], ds[b+1]) holds place q (ds ascending, ds[256] = values of the tile)
__device__ inline int route_digit_of(const uint32_t *ds, uint32_t q) {
    int b = 0;
#pragma unroll
    for (int step = 128; step >= 1; step >>= 1)
        if (ds[b + step] <= q) b += step;
    return b;
}

// pass 1 or 2 forwards: tile of `in` (tile order, in2 added if given) -> runs of `out`
__global__ __launch_bounds__(RT_NT) void route_deal_kernel(const float *__restrict__ in, const float *__restrict__ in2,
                                                           float *__restrict__ out, const uint16_t *__restrict__ slot,
                                                           const uint32_t *__restrict__ dstart_tab,
                                                           const uint32_t *__restrict__ gofs_tab, int B, int64_t n) {
    const int64_t tb = route_tile(n);
    if (tb < 0) return;
    __shared__ float stage[RT_TILE];
    __shared__ uint32_t ds[257], go[256];
    const int tid = threadIdx.x;
    const int64_t tile0 = tb * RT_TILE;
    const int64_t left = n - tile0;
    const int cnt = (int)(left < RT_TILE ? left : RT_TILE);
    if (tid <= 256) ds[tid] = dstart_tab[tb * 257 + tid];
    if (tid < 256) go[tid] = gofs_tab[tb * 256 + tid];
    uint16_t sl[RT_IPT];
    float v[RT_IPT];
#pragma unroll
    for (int r = 0; r < RT_IPT; ++r) {
        const int e = r * RT_NT + tid;
        sl[r] = e < cnt ? slot[tile0 + e] : (uint16_t)0;
        v[r] = e < cnt ? in[tile0 + e] : 0.f;
    }
    if (in2) {
#pragma unroll
        for (int r = 0; r < RT_IPT; ++r) {
            const int e = r * RT_NT + tid;
            if (e < cnt) v[r] += in2[tile0 + e];
        }
    }
#pragma unroll
    for (int r = 0; r < RT_IPT; ++r)
        if (r * RT_NT + tid < cnt) stage[sl[r]] = v[r];
    __syncthreads();
    // a thread per place: consecutive places of a run go to consecutive addresses, and all the stores of a
    // thread are independent (a wavefront per run would wait for one short run after the other)
#pragma unroll
    for (int r = 0; r < RT_IPT; ++r) {
        const uint32_t q = (uint32_t)(r * RT_NT + tid);
        if ((int)q < cnt) out[go[route_digit_of(ds, q)] + q] = stage[q];
    }
}

// pass 2 or 1 backwards: runs of `in` -> tile of `out` (tile order); NC components, one array each on the
// input side (in + c * in_stride); on the output side one array each (ROWS == false) or rows of NC values
template <int NC, bool ROWS>
__global__ __launch_bounds__(RT_NT) void route_collect_kernel(const float *__restrict__ in, int64_t in_stride,
                                                              float *__restrict__ out, int64_t out_stride,
                                                              const uint16_t *__restrict__ slot,
                                                              const uint32_t *__restrict__ dstart_tab,
                                                              const uint32_t *__restrict__ gofs_tab, int B, int64_t n) {
    const int64_t tb = route_tile(n);
    if (tb < 0) return;
    __shared__ float stage[RT_TILE];
    __shared__ uint32_t ds[257], go[256];
    const int tid = threadIdx.x;
    const int64_t tile0 = tb * RT_TILE;
    const int64_t left = n - tile0;
    const int cnt = (int)(left < RT_TILE ? left : RT_TILE);
    if (tid <= 256) ds[tid] = dstart_tab[tb * 257 + tid];
    if (tid < 256) go[tid] = gofs_tab[tb * 256 + tid];
    uint32_t sl[RT_IPT / 2];   // two places per register
#pragma unroll
    for (int r = 0; r < RT_IPT; r += 2) {
        const int e0 = r * RT_NT + tid, e1 = e0 + RT_NT;
        const uint32_t a = e0 < cnt ? slot[tile0 + e0] : 0u, b = e1 < cnt ? slot[tile0 + e1] : 0u;
        sl[r / 2] = a | (b << 16);
    }
    __syncthreads();
    float v[ROWS ? NC : 1][RT_IPT];
    // a thread per place (see route_deal_kernel): place q comes from go[digit of q] + q in the order before
    constexpr int FLY = ROWS ? 8 : 16;   // loads in flight per thread (the row variant is short of registers)
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const float *src = in + (int64_t)c * in_stride;
#pragma unroll
        for (int h = 0; h < RT_IPT; h += FLY) {
            float t[FLY];
#pragma unroll
            for (int r = 0; r < FLY; ++r) {
                const uint32_t q = (uint32_t)((h + r) * RT_NT + tid);
                t[r] = (int)q < cnt ? src[go[route_digit_of(ds, q)] + q] : 0.f;
            }
#pragma unroll
            for (int r = 0; r < FLY; ++r) stage[(h + r) * RT_NT + tid] = t[r];
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < RT_IPT; ++r) v[ROWS ? c : 0][r] = stage[(sl[r / 2] >> (16 * (r & 1))) & 0xFFFFu];
        if (!ROWS) {
            float *dst = out + (int64_t)c * out_stride;
#pragma unroll
            for (int r = 0; r < RT_IPT; ++r) {
                const int e = r * RT_NT + tid;
                if (e < cnt) dst[tile0 + e] = v[0][r];
            }
        }
        __syncthreads();
    }
    if (ROWS) {
        // a row leaves as one store of NC values
        struct Row { float v[NC]; };
        Row *rows = reinterpret_cast<Row *>(out);
#pragma unroll
        for (int r = 0; r < RT_IPT; ++r) {
            const int e = r * RT_NT + tid;
            if (e < cnt) {
                Row t;
#pragma unroll
                for (int c = 0; c < NC; ++c) t.v[c] = v[ROWS ? c : 0][r];
                rows[tile0 + e] = t;
            }
        }
    }
}

// pass 3 forwards: the values of a window, each to its place inside the window
__global__ __launch_bounds__(RT_NT) void route_place_kernel(const float *__restrict__ in, float *__restrict__ out,
                                                            const uint16_t *__restrict__ off, int64_t n) {
    const int64_t tb = route_tile(n);
    if (tb < 0) return;
    __shared__ float stage[RT_TILE];
    const int tid = threadIdx.x;
    const int64_t win0 = tb * RT_TILE;
    const int64_t left = n - win0;
    const int cnt = (int)(left < RT_TILE ? left : RT_TILE);
    uint16_t o[RT_IPT];
    float v[RT_IPT];
#pragma unroll
    for (int r = 0; r < RT_IPT; ++r) {
        const int e = r * RT_NT + tid;
        o[r] = e < cnt ? off[win0 + e] : (uint16_t)0;
        v[r] = e < cnt ? in[win0 + e] : 0.f;
    }
#pragma unroll
    for (int r = 0; r < RT_IPT; ++r)
        if (r * RT_NT + tid < cnt) stage[o[r]] = v[r];
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RT_IPT; ++r) {
        const int e = r * RT_NT + tid;
        if (e < cnt) out[win0 + e] = stage[e];
    }
}

// pass 3 backwards: a window of the caller's array (NC values per row, row-major) -> order p2, one array per
// component.  A thread reads its rows once, whole (the window of a point set is not read again per coordinate),
// and passes them through the LDS copy one coordinate at a time.
template <int NC>
__global__ __launch_bounds__(RT_NT) void route_pick_kernel(const float *__restrict__ in, float *__restrict__ out,
                                                           int64_t out_stride, const uint16_t *__restrict__ off,
                                                           int64_t n) {
    const int64_t tb = route_tile(n);
    if (tb < 0) return;
    __shared__ float stage[RT_TILE];
    const int tid = threadIdx.x;
    const int64_t win0 = tb * RT_TILE;
    const int64_t left = n - win0;
    const int cnt = (int)(left < RT_TILE ? left : RT_TILE);
    struct Row { float v[NC]; };
    Row row[RT_IPT];
    const Row *rows = reinterpret_cast<const Row *>(in);
#pragma unroll
    for (int r = 0; r < RT_IPT; ++r) {
        const int e = r * RT_NT + tid;
        row[r] = rows[win0 + (e < cnt ? e : 0)];
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int r = 0; r < RT_IPT; ++r) stage[r * RT_NT + tid] = row[r].v[c];
        __syncthreads();
        float *dst = out + (int64_t)c * out_stride;
#pragma unroll
        for (int h = 0; h < RT_IPT; h += 8) {
            uint32_t o[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int e = (h + r) * RT_NT + tid;
                o[r] = e < cnt ? off[win0 + e] : 0u;
            }
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int e = (h + r) * RT_NT + tid;
                if (e < cnt) dst[win0 + e] = stage[o[r]];
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------
static RouteLevel route_level(const f3m_route &R, int pass) {
    RouteLevel L{};
    L.second = pass == 2;
    L.s2 = R.s2;
    L.ntiles = R.ntiles;
    if (pass == 1) {
        L.shift = RT_BITS + R.s2;
        L.mask = 0xFFu;
        L.B = R.B1;
    } else {
        L.shift = RT_BITS;
        L.mask = (1u << R.s2) - 1u;
        L.B = R.B2;
    }
    return L;
}

// Tables of the three passes for the permutation perm (n entries, box order -> caller's index).
void route_build(f3m_route &R, const uint32_t *perm, int64_t n, int64_t *tally, hipStream_t st) {
    R.n = n;
    R.ntiles = cdiv(n, RT_TILE);
    int wbits = 0;
    while (((int64_t)1 << wbits) < R.ntiles) ++wbits;
    R.s2 = (wbits + 1) / 2;
    R.B2 = 1 << R.s2;
    R.B1 = (int)cdiv(R.ntiles, R.B2);
    if (R.B1 > 256 || R.B2 > 256) fail(F3M_ERR_UNSUPPORTED, "too many points for the three-pass permutation");
    R.slot1.alloc((size_t)n, tally);
    R.slot2.alloc((size_t)n, tally);
    R.off3.alloc((size_t)n, tally);
    R.dstart1.alloc((size_t)R.ntiles * 257, tally);
    R.dstart2.alloc((size_t)R.ntiles * 257, tally);
    R.gofs1.alloc((size_t)R.ntiles * 256, tally);
    R.gofs2.alloc((size_t)R.ntiles * 256, tally);
    DevBuf<uint32_t> dest1, cursor;
    dest1.alloc((size_t)n);
    const int64_t nwin = (int64_t)R.B1 * R.B2;   // windows, counting the empty ones behind the last value
    cursor.alloc((size_t)nwin);
    const unsigned grid = route_grid(R.ntiles);
    for (int pass = 1; pass <= 2; ++pass) {
        const RouteLevel L = route_level(R, pass);
        const uint32_t *din = pass == 1 ? perm : dest1.p;
        // first positions: bucket d1 at d1 B2 T, window w at w T
        const int64_t ncur = pass == 1 ? R.B1 : nwin;
        route_cursor_init_kernel<<<dim3((unsigned)cdiv(ncur, 256)), dim3(256), 0, st>>>(
            cursor.p, ncur, pass == 1 ? (uint32_t)R.B2 * (uint32_t)RT_TILE : (uint32_t)RT_TILE);
        route_rank_kernel<<<dim3(grid), dim3(RT_NT), 0, st>>>(din, n, L, cursor.p, pass == 1 ? R.slot1.p : R.slot2.p,
                                                             pass == 1 ? dest1.p : nullptr,
                                                             pass == 1 ? nullptr : R.off3.p,
                                                             pass == 1 ? R.dstart1.p : R.dstart2.p,
                                                             pass == 1 ? R.gofs1.p : R.gofs2.p);
        F3M_HIP(hipGetLastError());
    }
    F3M_HIP(hipStreamSynchronize(st));   // the work arrays are released on return
}

// out[perm[k]] = in[k] (+ in2[k]); tmp_a, tmp_b: n floats each
void route_scatter(const f3m_route &R, const float *in, const float *in2, float *out, float *tmp_a, float *tmp_b,
                   hipStream_t st) {
    const unsigned grid = route_grid(R.ntiles);
    route_deal_kernel<<<dim3(grid), dim3(RT_NT), 0, st>>>(in, in2, tmp_a, R.slot1.p, R.dstart1.p, R.gofs1.p, R.B1, R.n);
    route_deal_kernel<<<dim3(grid), dim3(RT_NT), 0, st>>>(tmp_a, nullptr, tmp_b, R.slot2.p, R.dstart2.p, R.gofs2.p, R.B2,
                                                         R.n);
    route_place_kernel<<<dim3(grid), dim3(RT_NT), 0, st>>>(tmp_b, out, R.off3.p, R.n);
    F3M_HIP(hipGetLastError());
}

// out[k] = in[perm[k]]; tmp_a, tmp_b: n floats each
void route_gather(const f3m_route &R, const float *in, float *out, float *tmp_a, float *tmp_b, hipStream_t st) {
    const unsigned grid = route_grid(R.ntiles);
    route_pick_kernel<1><<<dim3(grid), dim3(RT_NT), 0, st>>>(in, tmp_a, 0, R.off3.p, R.n);
    route_collect_kernel<1, false><<<dim3(grid), dim3(RT_NT), 0, st>>>(tmp_a, 0, tmp_b, 0, R.slot2.p, R.dstart2.p,
                                                                      R.gofs2.p, R.B2, R.n);
    route_collect_kernel<1, false><<<dim3(grid), dim3(RT_NT), 0, st>>>(tmp_b, 0, out, 0, R.slot1.p, R.dstart1.p,
                                                                      R.gofs1.p, R.B1, R.n);
    F3M_HIP(hipGetLastError());
}

// rows of three coordinates: out[k][0..2] = in[perm[k]][0..2].  `out` (3 n floats) first serves as the
// three component arrays of order p2; tmp: 3 n floats.
void route_gather_rows3(const f3m_route &R, const float *in, float *out, float *tmp, hipStream_t st) {
    const unsigned grid = route_grid(R.ntiles);
    route_pick_kernel<3><<<dim3(grid), dim3(RT_NT), 0, st>>>(in, out, R.n, R.off3.p, R.n);
    route_collect_kernel<3, false><<<dim3(grid), dim3(RT_NT), 0, st>>>(out, R.n, tmp, R.n, R.slot2.p, R.dstart2.p,
                                                                      R.gofs2.p, R.B2, R.n);
    route_collect_kernel<3, true><<<dim3(grid), dim3(RT_NT), 0, st>>>(tmp, R.n, out, 0, R.slot1.p, R.dstart1.p,
                                                                     R.gofs1.p, R.B1, R.n);
    F3M_HIP(hipGetLastError());
}

}  // namespace f3m
