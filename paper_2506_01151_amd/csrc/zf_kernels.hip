// HIP kernels for gfx950 around the mask kernels: the upload of the packed charts, the state cache's
// gather, and the logit-masking kernel.
//
// Mask path.  The distinct vocabulary strings are numbered in sorted order (their rank); verdicts
// are first produced in rank order.  The context-independent token-mask cache (Section 4.3) settles
// most strings from the terminals of the row's current Earley set alone; the strings it leaves
// undecided need the parser.  Two kernels can do that part (zf_options.walk_mode), both exact:
// the mask automaton (zf_mask_automaton.hip, default) and the trie walk (zf_mask_walk.hip, which
// also holds finish_kernel: the exact fallback pass of both, and the permutation of the verdicts
// into token order).
#include <hip/hip_runtime.h>
#include "zf_launch.h"

namespace zf {
namespace {

// The packed charts of a call, a few KB, from pinned host memory to device memory: launched like
// the kernels behind it (the runtime's copy path costs the host several times as long per call).
__global__ __launch_bounds__(256) void upload_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, uint32_t n16) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

// State cache (Section 5.2): copy every row's finished mask from its pool slot to the caller's
// tensor.  When the cache is on this is the call's last kernel.
__global__ __launch_bounds__(256) void gather_kernel(MaskArgs a) {
    const uint32_t w = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y, W = (uint32_t)a.tab.W;
    if (w < W) a.user_mask[(size_t)row * W + w] = a.out_mask[(size_t)a.row_slot[row] * W + w];
    // the block that is started last hands the counters to the host and clears the next call's set (see finish_kernel)
    if (blockIdx.x == gridDim.x - 1 && blockIdx.y == gridDim.y - 1) {
        __syncthreads();
        if (threadIdx.x < 8) a.counters_next[threadIdx.x] = 0;
        if (threadIdx.x == 0) {                           // counters first, then the word the host waits for
            for (int i = 0; i < 4; i++) a.host_status[i] = a.counters[i];
            if (a.store.ctl) for (int i = 0; i < 3; i++) a.host_status[5 + i] = a.store.ctl[i];
            __hip_atomic_store(&a.host_status[4], a.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

// Logit masking (Section 3.3): pure copy-or-(-inf).  16-byte accesses, consecutive lanes on
// consecutive 16-byte pieces; the mask words come from L2.
static const int APPLY_UNROLL = 4;   // 16-byte pieces per thread
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <typename VecT, int EPV /* elements per 16 bytes */, typename ElemT>
__global__ __launch_bounds__(256) void apply_mask_vec_kernel(const ElemT *__restrict__ in, ElemT *__restrict__ out, int64_t stride,
                                                             int V, int W, const uint32_t *__restrict__ mask, ElemT neg_inf) {
    const int row = blockIdx.y;
    const ElemT *src = in + (size_t)row * stride;
    ElemT *dst = out + (size_t)row * stride;
    const uint32_t *mrow = mask + (size_t)row * W;
    const int n_vec = V / EPV;
    // a block covers APPLY_UNROLL * 256 consecutive pieces: all loads of a thread are issued before its first store
    const int g0 = blockIdx.x * (256 * APPLY_UNROLL) + threadIdx.x;
    VecT x[APPLY_UNROLL];
#pragma unroll
    for (int u = 0; u < APPLY_UNROLL; u++) {
        const int g = g0 + u * 256;
        if (g < n_vec) x[u] = __builtin_nontemporal_load(reinterpret_cast<const VecT *>(src) + g);
    }
#pragma unroll
    for (int u = 0; u < APPLY_UNROLL; u++) {
        const int g = g0 + u * 256;
        if (g >= n_vec) break;
        const int v0 = g * EPV;
        const uint32_t mb = mrow[v0 >> 5] >> (v0 & 31);
        ElemT *e = reinterpret_cast<ElemT *>(&x[u]);
#pragma unroll
        for (int k = 0; k < EPV; k++) if (!((mb >> k) & 1u)) e[k] = neg_inf;
        __builtin_nontemporal_store(x[u], reinterpret_cast<VecT *>(dst) + g);
    }
    // ragged tail of the row
    const int t = n_vec * EPV + blockIdx.x * 256 + threadIdx.x;
    if (t < V && blockIdx.x * 256 + threadIdx.x < EPV) {
        const bool keep = (mrow[t >> 5] >> (t & 31)) & 1u;
        dst[t] = keep ? src[t] : neg_inf;
    }
}

template <typename ElemT>
__global__ __launch_bounds__(256) void apply_mask_scalar_kernel(const ElemT *__restrict__ in, ElemT *__restrict__ out, int64_t stride,
                                                                int V, int W, const uint32_t *__restrict__ mask, ElemT neg_inf) {
    const int row = blockIdx.y;
    for (int v = blockIdx.x * 256 + threadIdx.x; v < V; v += gridDim.x * 256) {
        const bool keep = (mask[(size_t)row * W + (v >> 5)] >> (v & 31)) & 1u;
        out[(size_t)row * stride + v] = keep ? in[(size_t)row * stride + v] : neg_inf;
    }
}

}  // namespace

hipError_t prepare_kernels() {
    hipError_t e = prepare_walk_kernels();
    if (e == hipSuccess) e = prepare_automaton_kernels();
    return e != hipSuccess ? e : prepare_store_kernels();
}

hipError_t launch_upload(const void *pinned_src, void *dst, size_t bytes, hipStream_t s) {
    const uint32_t n16 = (uint32_t)((bytes + 15) / 16);
    hipLaunchKernelGGL(upload_kernel, dim3((n16 + 255) / 256), dim3(256), 0, s, (const uint4 *)pinned_src, (uint4 *)dst, n16);
    return hipGetLastError();
}
hipError_t launch_gather(const MaskArgs &a, hipStream_t s) {
    dim3 grid((a.tab.W + 255) / 256 > 0 ? (a.tab.W + 255) / 256 : 1, a.user_batch);
    hipLaunchKernelGGL(gather_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_apply_mask(const void *logits, void *out, int dtype, int batch, int64_t row_stride, int V, int W,
                             const uint32_t *mask, hipStream_t s) {
    const size_t esz = dtype == 0 ? 4 : 2;
    const bool aligned = ((uintptr_t)logits % 16 == 0) && ((uintptr_t)out % 16 == 0) && ((row_stride * esz) % 16 == 0);
    const int epv = (int)(16 / esz);
    int blocks_x = aligned ? (V / epv + 256 * APPLY_UNROLL - 1) / (256 * APPLY_UNROLL) : (V + 255) / 256;
    if (blocks_x < 1) blocks_x = 1;
    dim3 grid(blocks_x, batch);
    if (dtype == 0) {
        const uint32_t ninf = 0xFF800000u;
        if (aligned) hipLaunchKernelGGL((apply_mask_vec_kernel<u32x4, 4, uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)logits, (uint32_t *)out, row_stride, V, W, mask, ninf);
        else hipLaunchKernelGGL((apply_mask_scalar_kernel<uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)logits, (uint32_t *)out, row_stride, V, W, mask, ninf);
    } else {
        const uint16_t ninf = 0xFF80u;
        if (aligned) hipLaunchKernelGGL((apply_mask_vec_kernel<u32x4, 8, uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)logits, (uint16_t *)out, row_stride, V, W, mask, ninf);
        else hipLaunchKernelGGL((apply_mask_scalar_kernel<uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)logits, (uint16_t *)out, row_stride, V, W, mask, ninf);
    }
    return hipGetLastError();
}

}  // namespace zf
