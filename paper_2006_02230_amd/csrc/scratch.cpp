// Device scratch memory the split-reduction kernels use: per (device, stream) one buffer for the
// partial accumulator tiles and one array of arrival counters.  Work on one stream is ordered, so
// consecutive launches on it may share a buffer; launches on different streams get different ones.
#include <hip/hip_runtime.h>
#include <map>
#include <mutex>
#include <utility>
#include "internal.hpp"

namespace polydl {

namespace {
struct Scratch {
    float *partials = nullptr;
    size_t partial_bytes = 0;
    unsigned *counters = nullptr;
    int ncounters = 0;
};
std::mutex g_scratch_mu;
std::map<std::pair<int, hipStream_t>, Scratch> g_scratch;
}  // namespace

// Returns buffers of at least partial_bytes bytes and tiles counters (all zero: every kernel
// leaves the counters it used at zero again).  Buffers only grow; growing frees the old buffer,
// which waits for the device, so no running kernel loses its memory.
hipError_t splitk_scratch(hipStream_t stream, size_t partial_bytes, int tiles, float **partials, unsigned **counters)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    Scratch &s = g_scratch[std::make_pair(dev, stream)];
    if (s.partial_bytes < partial_bytes) {
        if (s.partials) {
            e = hipFree(s.partials);
            s.partials = nullptr;
            s.partial_bytes = 0;
            if (e != hipSuccess) return e;
        }
        // a quarter more than asked, so a run of slightly growing problems does not reallocate each time
        size_t want = partial_bytes + partial_bytes / 4;
        want = (want + 255) & ~(size_t)255;
        e = hipMalloc(reinterpret_cast<void **>(&s.partials), want);
        if (e != hipSuccess) { s.partials = nullptr; return e; }
        s.partial_bytes = want;
    }
    if (s.ncounters < tiles) {
        if (s.counters) {
            e = hipFree(s.counters);
            s.counters = nullptr;
            s.ncounters = 0;
            if (e != hipSuccess) return e;
        }
        int want = tiles < 4096 ? 4096 : tiles + tiles / 4;
        e = hipMalloc(reinterpret_cast<void **>(&s.counters), (size_t)want * sizeof(unsigned));
        if (e != hipSuccess) { s.counters = nullptr; return e; }
        e = hipMemset(s.counters, 0, (size_t)want * sizeof(unsigned));   // synchronous: done before any launch
        if (e != hipSuccess) return e;
        s.ncounters = want;
    }
    *partials = s.partials;
    *counters = s.counters;
    return hipSuccess;
}

// Compute units of the current device (asked once per device).
int compute_units()
{
    static std::map<int, int> cus;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    auto it = cus.find(dev);
    if (it != cus.end()) return it->second;
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    cus[dev] = n;
    return n;
}

}  // namespace polydl
