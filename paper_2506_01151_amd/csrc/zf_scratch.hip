// Device memory of the entry point that may not allocate (zf_compute_mask_noalloc): one static
// device array per GPU, present from the moment the library is loaded on that GPU until the
// process ends.  Every per-call buffer of such a call (counters, rank-ordered verdict words, the
// fallback list and arenas, the trie walk's queue, the device copy of the packed charts) is a
// slice of it.  All calls on one GPU share the array and it keeps the last call's contents: the
// call clears what must start at zero, and calls that overlap on one GPU race.
#include <hip/hip_runtime.h>
#include <mutex>
#include "zf_launch.h"

namespace zf {
namespace {

static __device__ __align__(256) __attribute__((used)) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

// In host code the array's name is only a handle for the runtime; the memory's address on a
// given GPU comes from hipGetSymbolAddress with that GPU current, and differs from GPU to GPU.
const int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

__global__ __launch_bounds__(256) void clear_words_kernel(uint32_t *p, uint32_t n) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace

hipError_t scratch_init(int device) {
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (g_scratch_ptr[device]) return hipSuccess;
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = p;
    return hipSuccess;
}

void *scratch_ptr(int device) {
    if (device < 0 || device >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    return g_scratch_ptr[device];
}

hipError_t launch_clear_words(uint32_t *p, uint32_t n_words, hipStream_t s) {
    if (n_words == 0) return hipSuccess;
    hipLaunchKernelGGL(clear_words_kernel, dim3((n_words + 255) / 256), dim3(256), 0, s, p, n_words);
    return hipGetLastError();
}

}  // namespace zf
