// Device memory of the library comes from a small caching pool: a buffer that is released goes back
// to the pool and the next request of the same size class gets it again.  A plan for n = 1e9 points
// holds ~57 GB in some sixty buffers; building plan after plan (one per time step of a solver, one per
// benchmark step) otherwise pays hipMalloc / hipFree for all of them every time, and on a device
// whose memory was just given back by another process an allocation can take tens of milliseconds
// per gigabyte.  A release waits for the device before the block is put back (as hipFree would), so a
// block is never handed out again while work that uses it is still in flight, on whatever stream.
#include <map>
#include <mutex>

#include "common.h"

namespace f3m {
namespace {

struct Pool {
    std::mutex m;
    std::multimap<std::pair<int, size_t>, void *> blocks;   // (device, class size) -> free block
    size_t held = 0;                                          // bytes of the free blocks
};
Pool &pool() {
    static Pool *p = new Pool();   // never destroyed: the HIP runtime may be gone at process exit
    return *p;
}
constexpr size_t POOL_CAP = (size_t)96 << 30;   // free blocks beyond this are given back to the device

// size classes: multiples of 1/16 of the power of two below the size (at most 6.25 % over)
size_t class_size(size_t bytes) {
    if (bytes < 4096) return 4096;
    int lg = 63 - __builtin_clzll((unsigned long long)bytes);
    const size_t g = (size_t)1 << (lg - 4);
    return (bytes + g - 1) / g * g;
}

size_t trim_locked(Pool &P, size_t keep) {
    size_t freed = 0;
    // largest blocks first
    while (P.held > keep && !P.blocks.empty()) {
        auto it = P.blocks.begin(), best = it;
        for (; it != P.blocks.end(); ++it)
            if (it->first.second > best->first.second) best = it;
        (void)hipFree(best->second);
        P.held -= best->first.second;
        freed += best->first.second;
        P.blocks.erase(best);
    }
    return freed;
}

}  // namespace

void *pool_alloc(size_t bytes) {
    const size_t cs = class_size(bytes);
    int dev = 0;
    F3M_HIP(hipGetDevice(&dev));
    Pool &P = pool();
    {
        std::lock_guard<std::mutex> lock(P.m);
        auto it = P.blocks.find({dev, cs});
        if (it != P.blocks.end()) {
            void *p = it->second;
            P.blocks.erase(it);
            P.held -= cs;
            return p;
        }
    }
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, cs);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        pool_trim();   // give the cached blocks back and try once more
        e = hipMalloc(&p, cs);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        fail(F3M_ERR_OOM, "hipMalloc of " + std::to_string(cs) + " bytes failed: " + hipGetErrorString(e));
    }
    return p;
}

void pool_free(void *p, size_t bytes) {
    if (!p) return;
    const size_t cs = class_size(bytes);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(p);
        return;
    }
    (void)hipDeviceSynchronize();   // nothing in flight may still use the block
    Pool &P = pool();
    std::lock_guard<std::mutex> lock(P.m);
    P.blocks.insert({{dev, cs}, p});
    P.held += cs;
    if (P.held > POOL_CAP) trim_locked(P, POOL_CAP);
}

size_t pool_trim() {
    Pool &P = pool();
    std::lock_guard<std::mutex> lock(P.m);
    return trim_locked(P, 0);
}

}  // namespace f3m
