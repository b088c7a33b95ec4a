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
#include <algorithm>
#include "zf_kernel_common.h"


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
    hand_over(a, blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y, false);   // the call's last kernel when the state cache is on; nothing in it can fail
}

// Logit masking (Section 3.3): pure copy-or-(-inf).  The tensor is taken as one run of 16-byte pieces (rows x pieces per
// row), consecutive lanes on consecutive pieces, so that no block is left with the thin end of a row; a thread has U
// pieces in flight (all loads issued before the first store); loads and stores are non-temporal; the mask words come
// from L2.  `in` and `out` may be the same tensor (each thread reads its pieces before it writes them), so neither is
// declared restrict.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <int EPV /* elements per 16 bytes */, int U, typename ElemT>
__global__ __launch_bounds__(256) void apply_mask_vec_kernel(const ElemT *in, ElemT *out, int64_t stride, int V, int W, int batch,
                                                             const uint32_t *__restrict__ mask, ElemT neg_inf) {
    const uint32_t n_vec = (uint32_t)V / EPV;                 // whole pieces per row
    const uint32_t total = n_vec * (uint32_t)batch;           // the host checks that this fits 32 bits
    const uint32_t g0 = blockIdx.x * (256 * U) + threadIdx.x;
    u32x4 x[U];
    uint32_t row[U], col[U];
    uint32_t r = g0 / n_vec, c = g0 - r * n_vec;              // one division per thread; the later pieces by stepping
#pragma unroll
    for (int u = 0; u < U; u++) {
        row[u] = r; col[u] = c;
        if (g0 + (uint32_t)u * 256 < total) x[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(in + (size_t)r * stride) + c);
        c += 256;
        while (c >= n_vec) { c -= n_vec; r++; }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
        if (g0 + (uint32_t)u * 256 >= total) break;
        const uint32_t v0 = col[u] * EPV;
        const uint32_t mb = mask[(size_t)row[u] * W + (v0 >> 5)] >> (v0 & 31);
        ElemT *e = reinterpret_cast<ElemT *>(&x[u]);
#pragma unroll
        for (int k = 0; k < EPV; k++) if (!((mb >> k) & 1u)) e[k] = neg_inf;
        __builtin_nontemporal_store(x[u], reinterpret_cast<u32x4 *>(out + (size_t)row[u] * stride) + col[u]);
    }
    // ragged tails of the rows (V not a multiple of the piece): the first threads of the grid, one element each
    const uint32_t tail = (uint32_t)V - n_vec * EPV;
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (tail && t < (uint64_t)tail * (uint32_t)batch) {
        const uint32_t r = (uint32_t)(t / tail), v = n_vec * EPV + (uint32_t)(t - (uint64_t)r * tail);
        const bool keep = (mask[(size_t)r * W + (v >> 5)] >> (v & 31)) & 1u;
        out[(size_t)r * stride + v] = keep ? in[(size_t)r * stride + v] : neg_inf;
    }
}

template <typename ElemT>
__global__ __launch_bounds__(256) void apply_mask_scalar_kernel(const ElemT *in, ElemT *out, int64_t stride,
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

template <int EPV, typename ElemT>
static void launch_apply_vec(const ElemT *in, ElemT *out, int64_t stride, int V, int W, int batch, const uint32_t *mask, ElemT ninf, hipStream_t s) {
    // Pieces in flight per thread by the size of the tensor: a small one needs many blocks to reach every compute unit at all,
    // a larger one more bytes in flight per wavefront to cover the memory latency (8 TB/s x 2 us = 16 MB on the way).
    const uint64_t total = (uint64_t)(V / EPV) * (uint64_t)batch;
    const uint64_t tail = (uint64_t)(V % EPV) * (uint64_t)batch;
    auto blocks = [&](int u) { return (uint32_t)std::max<uint64_t>(std::max<uint64_t>((total + 256ull * u - 1) / (256ull * u), (tail + 255) / 256), 1); };
    // measured on [16..1024] x 128,256 bf16 / fp32 and [64] x 152,064 fp32 (kernel-trace durations): the differences are a few per cent
    if (total >= (1ull << 22)) hipLaunchKernelGGL((apply_mask_vec_kernel<EPV, 2, ElemT>), dim3(blocks(2)), dim3(256), 0, s, in, out, stride, V, W, batch, mask, ninf);
    else if (total >= (1ull << 20)) hipLaunchKernelGGL((apply_mask_vec_kernel<EPV, 8, ElemT>), dim3(blocks(8)), dim3(256), 0, s, in, out, stride, V, W, batch, mask, ninf);
    else if (total >= (1ull << 18)) hipLaunchKernelGGL((apply_mask_vec_kernel<EPV, 4, ElemT>), dim3(blocks(4)), dim3(256), 0, s, in, out, stride, V, W, batch, mask, ninf);
    else hipLaunchKernelGGL((apply_mask_vec_kernel<EPV, 1, ElemT>), dim3(blocks(1)), dim3(256), 0, s, in, out, stride, V, W, batch, mask, ninf);
}

hipError_t launch_apply_mask(const void *logits, void *out, int dtype, int batch, int64_t row_stride, int V, int W,
                             const uint32_t *mask, hipStream_t s) {
    const size_t esz = dtype == 0 ? 4 : 2;
    const bool aligned = ((uintptr_t)logits % 16 == 0) && ((uintptr_t)out % 16 == 0) && ((row_stride * esz) % 16 == 0) &&
                         (uint64_t)V * (uint64_t)batch < (1ull << 32) && (uint64_t)V / (16 / esz) > 0;
    dim3 grid((V + 255) / 256 > 0 ? (V + 255) / 256 : 1, batch);
    if (dtype == 0) {
        const uint32_t ninf = 0xFF800000u;
        if (aligned) launch_apply_vec<4, uint32_t>((const uint32_t *)logits, (uint32_t *)out, row_stride, V, W, batch, mask, ninf, s);
        else hipLaunchKernelGGL((apply_mask_scalar_kernel<uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)logits, (uint32_t *)out, row_stride, V, W, mask, ninf);
    } else {
        const uint16_t ninf = 0xFF80u;
        if (aligned) launch_apply_vec<8, uint16_t>((const uint16_t *)logits, (uint16_t *)out, row_stride, V, W, batch, mask, ninf, s);
        else hipLaunchKernelGGL((apply_mask_scalar_kernel<uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)logits, (uint16_t *)out, row_stride, V, W, mask, ninf);
    }
    return hipGetLastError();
}

}  // namespace zf
