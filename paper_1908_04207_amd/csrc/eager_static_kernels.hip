// The library's fixed scratch memory, for callers that cannot allocate device memory (code
// under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The
// statistics workspace that eager_stats_attach takes from the caller lives here as one
// file-scope device array of a fixed size; every GPU the library runs on holds its own copy
// until the process ends.  In host code the array's name is only a stand-in for the symbol:
// its device address is looked up once per device with hipGetSymbolAddress, and that pointer -
// never the name - is what kernels and the host side get.
#include "eager_internal.h"

#include <mutex>

namespace eager {
namespace {

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;

// One block of table entries from the kernel-argument segment to the table in the scratch.
__global__ __launch_bounds__(256) void table_fill_kernel(const TableArgs a)
{
    const int t = static_cast<int>(threadIdx.x);
    if (t < 2 * a.count) a.table[2 * static_cast<long long>(a.first) + t] = a.start_end[t];
}

}  // namespace

hipError_t static_scratch(char **ptr)
{
    static std::mutex mu;
    static char *per_device[kMaxDevices] = {};
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void *p = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = static_cast<char *>(p);
    }
    *ptr = per_device[dev];
    return hipSuccess;
}

hipError_t launch_table_fill(long long *table, const long long *start_end, int n_buckets,
                             hipStream_t stream)
{
    static_assert(2 * kTableChunk <= 256, "one thread per table entry");
    for (int first = 0; first < n_buckets; first += kTableChunk) {
        TableArgs a;
        a.table = table;
        a.first = first;
        a.count = n_buckets - first < kTableChunk ? n_buckets - first : kTableChunk;
        for (int i = 0; i < 2 * a.count; ++i) a.start_end[i] = start_end[2 * first + i];
        for (int i = 2 * a.count; i < 2 * kTableChunk; ++i) a.start_end[i] = 0;
        hipLaunchKernelGGL(table_fill_kernel, dim3(1), dim3(256), 0, stream, a);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace eager
