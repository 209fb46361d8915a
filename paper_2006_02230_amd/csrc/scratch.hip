// Device scratch memory of the split-reduction kernels: partial accumulator tiles and one arrival
// counter per tile.  Two sources:
//   * buffers the library allocates per (device, stream).  Work on one stream is ordered, so
//     consecutive launches on it may share a buffer; launches on different streams get different
//     ones.  A buffer that has been handed out is never freed: a larger one is allocated beside
//     it and the old one stays valid for launches recorded earlier (a captured graph keeps the
//     addresses it was recorded with);
//   * one fixed array in the code object (`scratch` below), for the entry point that may not
//     allocate.  Every device the library runs on holds its own copy for the life of the process.
#include <hip/hip_runtime.h>
#include <map>
#include <mutex>
#include <utility>
#include <vector>
#include "internal.hpp"

namespace polydl {

// The fixed array: counters first, partial tiles behind them.  In host code this name is only a
// handle for hipGetSymbolAddress; the device address is asked for once per device and used from
// then on.
static __device__ __align__(256) unsigned char scratch[kStaticCounterBytes + kStaticPartialBytes];

__global__ void zero_words_kernel(unsigned *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

namespace {
struct Scratch {
    float *partials = nullptr;
    size_t partial_bytes = 0;
    unsigned *counters = nullptr;
    int ncounters = 0;
    std::vector<void *> retired;   // smaller buffers handed out earlier, kept until the process ends
};
std::mutex g_scratch_mu;
std::map<std::pair<int, hipStream_t>, Scratch> g_scratch;
std::map<int, unsigned char *> g_static_base;   // device -> address of that device's copy of `scratch`
thread_local int t_refusal = SCRATCH_OK;

bool capturing(hipStream_t stream)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}
}  // namespace

int scratch_refusal() { return t_refusal; }

hipError_t static_scratch_arena(ScratchArena *arena)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    auto it = g_static_base.find(dev);
    if (it == g_static_base.end()) {
        unsigned char *base = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&base), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!base) return hipErrorInvalidSymbol;
        it = g_static_base.emplace(dev, base).first;
    }
    arena->counters = reinterpret_cast<unsigned *>(it->second);
    arena->ncounters = (int)(kStaticCounterBytes / sizeof(unsigned));
    arena->partials = reinterpret_cast<float *>(it->second + kStaticCounterBytes);
    arena->partial_bytes = kStaticPartialBytes;
    arena->clear_counters = true;
    return hipSuccess;
}

// Buffers of at least partial_bytes bytes and `tiles` counters, all counters zero (every kernel
// leaves the counters it used at zero again).
hipError_t splitk_scratch(hipStream_t stream, const ScratchArena *arena, size_t partial_bytes, int tiles,
                          float **partials, unsigned **counters)
{
    t_refusal = SCRATCH_OK;
    if (arena) {
        if (partial_bytes > arena->partial_bytes || tiles > arena->ncounters) {
            t_refusal = SCRATCH_TOO_SMALL;
            return hipErrorOutOfMemory;
        }
        *partials = arena->partials;
        *counters = arena->counters;
        if (arena->clear_counters) {
            // the array is shared by every call on this device and keeps what the last one left:
            // a launch that did not run to its end may have left counts behind
            return launch_kernel(zero_words_kernel, dim3((unsigned)((tiles + 255) / 256)), dim3(256), 0, stream,
                                 arena->counters, tiles);
        }
        return hipSuccess;
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    Scratch &s = g_scratch[std::make_pair(dev, stream)];
    const bool grow = s.partial_bytes < partial_bytes || s.ncounters < tiles;
    if (grow && capturing(stream)) {
        // allocation and the synchronous clear are not allowed while the stream is being captured
        t_refusal = SCRATCH_CAPTURING;
        return hipErrorStreamCaptureUnsupported;
    }
    if (s.partial_bytes < partial_bytes) {
        // a quarter more than asked, so a run of slightly growing problems does not reallocate each time
        size_t want = partial_bytes + partial_bytes / 4;
        want = (want + 255) & ~(size_t)255;
        float *fresh = nullptr;
        e = hipMalloc(reinterpret_cast<void **>(&fresh), want);
        if (e != hipSuccess) return e;
        if (s.partials) s.retired.push_back(s.partials);
        s.partials = fresh;
        s.partial_bytes = want;
    }
    if (s.ncounters < tiles) {
        int want = tiles < 4096 ? 4096 : tiles + tiles / 4;
        unsigned *fresh = nullptr;
        e = hipMalloc(reinterpret_cast<void **>(&fresh), (size_t)want * sizeof(unsigned));
        if (e != hipSuccess) return e;
        e = hipMemset(fresh, 0, (size_t)want * sizeof(unsigned));   // synchronous: done before any launch
        if (e != hipSuccess) { (void)hipFree(fresh); return e; }
        if (s.counters) s.retired.push_back(s.counters);
        s.counters = fresh;
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
