// Internal declarations shared by the HIP sources of libf3m (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <string>
#include <type_traits>
#include <vector>

#include "../../include/f3m.h"

namespace f3m {

struct Error {
    f3m_status status;
    std::string msg;
};

[[noreturn]] inline void fail(f3m_status st, const std::string &msg) { throw Error{st, msg}; }

#define F3M_HIP(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) {                                                               \
            (void)hipGetLastError(); /* reported here: the next call must not find it again */ \
            ::f3m::fail(e_ == hipErrorOutOfMemory ? F3M_ERR_OOM : F3M_ERR_HIP,                \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                   \
        }                                                                                     \
    } while (0)

// pool.hip: device memory through a caching pool (released blocks are kept for the next request of
// the same size class; pool_trim gives them back to the device and returns the bytes freed)
void *pool_alloc(size_t bytes);
void pool_free(void *p, size_t bytes);
size_t pool_trim();

// A device allocation that releases itself; the byte count is added to *tally if given.
template <class T>
struct DevBuf {
    T *p = nullptr;
    size_t count = 0;
    int64_t *tally = nullptr;
    DevBuf() = default;
    DevBuf(const DevBuf &) = delete;
    DevBuf &operator=(const DevBuf &) = delete;
    DevBuf(DevBuf &&o) noexcept : p(o.p), count(o.count), tally(o.tally) { o.p = nullptr; o.count = 0; }
    DevBuf &operator=(DevBuf &&o) noexcept {
        if (this != &o) { release(); p = o.p; count = o.count; tally = o.tally; o.p = nullptr; o.count = 0; }
        return *this;
    }
    ~DevBuf() { release(); }
    void alloc(size_t n, int64_t *tally_ = nullptr) {
        release();
        tally = tally_;
        count = n;
        size_t bytes = (n ? n : 1) * sizeof(T);
        p = nullptr;
        try {
            p = (T *)pool_alloc(bytes);
        } catch (...) {
            count = 0;
            throw;
        }
        if (tally) *tally += (int64_t)bytes;
    }
    void release() {
        if (p) {
            pool_free(p, (count ? count : 1) * sizeof(T));
            if (tally) *tally -= (int64_t)((count ? count : 1) * sizeof(T));
        }
        p = nullptr; count = 0;
    }
};

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------------------------------
// device-wide exclusive prefix sum (reduce, scan the block sums recursively, apply): no
// spinning, no cross-block dependence inside a kernel.
//   In :  __device__ uint64_t operator()(int64_t i) const      value of element i
//   Out:  __device__ void operator()(int64_t i, uint64_t exclusive, uint64_t value) const
// ---------------------------------------------------------------------------------------
constexpr int SCAN_NT = 256;
constexpr int SCAN_IPT = 8;
constexpr int SCAN_TILE = SCAN_NT * SCAN_IPT;

// inclusive running sum over the 64 lanes of a wavefront, every lane active: four shifts inside the
// rows of 16 lanes, then the row totals are passed on (lane 15 of a row to the next row, lane 31 to
// the upper half); a lane outside the source range adds zero
__device__ inline uint32_t wave_incl_scan_u32(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ inline uint64_t wave_incl_scan_u64(uint64_t v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint64_t t = __shfl_up(v, off, 64);
        if (lane >= off) v += t;
    }
    return v;
}

// exclusive scan of one value per thread over a 256-thread block; *total = block sum
__device__ inline uint64_t block_excl_scan_u64(uint64_t v, uint64_t *total) {
    __shared__ uint64_t wsum[SCAN_NT / 64];
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint64_t incl = wave_incl_scan_u64(v, lane);
    __syncthreads();  // protects wsum against a previous use
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    uint64_t base = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < SCAN_NT / 64; ++k) {
        uint64_t s = wsum[k];
        if (k < w) base += s;
        tot += s;
    }
    *total = tot;
    return base + incl - v;
}

// The SCAN_IPT consecutive inputs of a thread (zero behind the end).  An input type may hand over a whole run
// at once (load_run(base, v), base a multiple of SCAN_IPT, all of the run inside the array): it can then read
// its array with a few wide loads instead of one dependent narrow load per input.
template <class T, class = void>
struct has_load_run : std::false_type {};
template <class T>
struct has_load_run<T, std::void_t<decltype(&T::load_run)>> : std::true_type {};
template <class In>
__device__ inline void scan_load(const In &in, int64_t base, int64_t n, uint64_t (&v)[SCAN_IPT]) {
    if constexpr (has_load_run<In>::value) {
        if (base + SCAN_IPT <= n) {
            in.load_run(base, v);
            return;
        }
    }
#pragma unroll
    for (int k = 0; k < SCAN_IPT; ++k) v[k] = (base + k < n) ? in(base + k) : 0;
}

template <class In>
__global__ __launch_bounds__(SCAN_NT) void scan_reduce_kernel(In in, int64_t n, uint64_t *block_sums) {
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_IPT;
    uint64_t v[SCAN_IPT];
    scan_load(in, base, n, v);
    uint64_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_IPT; ++k) s += v[k];
    uint64_t tot;
    block_excl_scan_u64(s, &tot);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = tot;
}

template <class In, class Out>
__global__ __launch_bounds__(SCAN_NT) void scan_apply_kernel(In in, int64_t n, const uint64_t *block_offsets, Out out) {
    int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_IPT;
    uint64_t v[SCAN_IPT];
    scan_load(in, base, n, v);
    uint64_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_IPT; ++k) s += v[k];
    uint64_t tot;
    uint64_t ex = block_excl_scan_u64(s, &tot) + (block_offsets ? block_offsets[blockIdx.x] : 0);
#pragma unroll
    for (int k = 0; k < SCAN_IPT; ++k) {
        if (base + k < n) out(base + k, ex, v[k]);
        ex += v[k];
    }
}

struct ArrayInU64 {
    const uint64_t *p;
    __device__ uint64_t operator()(int64_t i) const { return p[i]; }
};
struct ArrayOutU64 {
    uint64_t *p;
    __device__ void operator()(int64_t i, uint64_t ex, uint64_t) const { p[i] = ex; }
};

// Exclusive scan of n elements in two host steps, so that the caller can size the output
// from the grand total before the values are written.
struct ScanState {
    DevBuf<uint64_t> sums;  // scanned block sums
    int64_t nblk = 0;
    uint64_t total = 0;
};

template <class In>
void scan_prepare(In in, int64_t n, ScanState &S, bool want_total, hipStream_t st);

template <class In, class Out>
void scan_finish(In in, int64_t n, ScanState &S, Out out, hipStream_t st) {
    if (n <= 0) return;
    scan_apply_kernel<<<dim3((unsigned)S.nblk), dim3(SCAN_NT), 0, st>>>(in, n, (const uint64_t *)S.sums.p, out);
    F3M_HIP(hipGetLastError());
}

template <class In>
void scan_prepare(In in, int64_t n, ScanState &S, bool want_total, hipStream_t st) {
    S.total = 0;
    S.nblk = 0;
    if (n <= 0) return;
    S.nblk = cdiv(n, SCAN_TILE);
    S.sums.alloc((size_t)S.nblk + 1);
    scan_reduce_kernel<<<dim3((unsigned)S.nblk), dim3(SCAN_NT), 0, st>>>(in, n, S.sums.p);
    F3M_HIP(hipGetLastError());
    if (S.nblk == 1) {
        if (want_total) {
            F3M_HIP(hipMemcpyAsync(&S.total, S.sums.p, sizeof(uint64_t), hipMemcpyDeviceToHost, st));
            F3M_HIP(hipStreamSynchronize(st));
        }
        F3M_HIP(hipMemsetAsync(S.sums.p, 0, sizeof(uint64_t), st));
        return;
    }
    // scan the block sums in place; the grand total of that scan is the grand total
    ScanState inner;
    scan_prepare(ArrayInU64{S.sums.p}, S.nblk, inner, want_total, st);
    scan_finish(ArrayInU64{S.sums.p}, S.nblk, inner, ArrayOutU64{S.sums.p}, st);
    S.total = inner.total;
    F3M_HIP(hipStreamSynchronize(st));  // `inner` is released on return
}

template <class In, class Out>
void exclusive_scan(In in, int64_t n, Out out, uint64_t *total_host, hipStream_t st) {
    ScanState S;
    scan_prepare(in, n, S, total_host != nullptr, st);
    scan_finish(in, n, S, out, st);
    if (total_host) *total_host = S.total;
    if (n > 0) F3M_HIP(hipStreamSynchronize(st));  // S.sums is released on return
}

}  // namespace f3m
