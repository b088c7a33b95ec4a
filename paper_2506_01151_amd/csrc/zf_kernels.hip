// HIP kernels for gfx950: the vocabulary-mask kernel (main pass + exact fallback pass), the
// rank-order -> token-order bit permutation, and the logit-masking kernel.
//
// Mask kernel.  The vocabulary trie is stored in preorder, so a depth-first walk is a linear
// scan in which a dead subtree is left through the node's skip pointer and a shared prefix is
// scanned once per lane.  Every lane owns the nodes of CHUNK_RANKS consecutive strings (one
// 32-bit word of verdicts).  It first replays the ancestors of its first node, then walks its
// nodes; per node it performs one Earley byte step (Scan + Complete with tabulated Predict,
// paper Section 3.2) on a private item list kept in LDS, interleaved by lane so that lanes
// never collide on a bank.  The list holds one set per trie depth of the current path; moving
// to a shallower node simply truncates it.  A lane whose list would outgrow its budget (or
// whose path is too deep) reports its chunk to the fallback pass, which repeats the same walk
// with the list in a global-memory arena.
#include <hip/hip_runtime.h>
#include "zf_launch.h"

namespace zf {
namespace {

struct LdsStore {
    uint2 *items;     // this lane's column of the block's item array (stride 64)
    uint8_t *ss;      // this lane's column of the set-start array (stride 64)
    uint32_t cap;
    static constexpr int max_depth = LANE_DEPTH_MAX;
    __device__ __forceinline__ uint2 get(uint32_t i) const { return items[i * 64]; }
    __device__ __forceinline__ void put(uint32_t i, uint2 v) { items[i * 64] = v; }
    __device__ __forceinline__ uint32_t start(int d) const { return ss[d * 64]; }
    __device__ __forceinline__ void set_start(int d, uint32_t v) { ss[d * 64] = (uint8_t)v; }
};

struct GlobalStore {
    uint2 *items;     // this lane's column of the arena (stride FB_LANES)
    uint32_t *ss;
    uint32_t cap;
    static constexpr int max_depth = FB_DEPTH_MAX;
    __device__ __forceinline__ uint2 get(uint32_t i) const { return items[(size_t)i * FB_LANES]; }
    __device__ __forceinline__ void put(uint32_t i, uint2 v) { items[(size_t)i * FB_LANES] = v; }
    __device__ __forceinline__ uint32_t start(int d) const { return ss[(size_t)d * FB_LANES]; }
    __device__ __forceinline__ void set_start(int d, uint32_t v) { ss[(size_t)d * FB_LANES] = v; }
};

// items are uint2: x = dotted position | DFA state << 16, y = origin set
template <class S>
__device__ __forceinline__ bool insert_unique(S &st, uint32_t set_begin, uint32_t &cnt, uint32_t pq, uint32_t o) {
    for (uint32_t i = set_begin; i < cnt; i++) {
        uint2 x = st.get(i);
        if (x.x == pq && x.y == o) return true;
    }
    if (cnt >= st.cap) return false;
    st.put(cnt++, make_uint2(pq, o));
    return true;
}

// Add the item with the dot at position p; skip nullable postdot nonterminals; record a dot at
// the end of a rule as the canonical "lhs complete since o" item.
template <class S>
__device__ __forceinline__ bool add_advanced(const DeviceTables &T, S &st, uint32_t set_begin, uint32_t &cnt, uint32_t p, uint32_t o) {
    for (;;) {
        uint32_t code = T.sym[p];
        uint32_t k = code >> SYM_KIND_SHIFT;
        if (k == SYM_END) return insert_unique(st, set_begin, cnt, T.end_pos[code & SYM_ID_MASK], o);
        if (k == SYM_TERM) return insert_unique(st, set_begin, cnt, p | ((uint32_t)T.term_start[code & SYM_ID_MASK] << 16), o);
        if (!insert_unique(st, set_begin, cnt, p, o)) return false;
        if (!(code & SYM_NULLABLE_BIT)) return true;
        p++;
    }
}

enum { STEP_ALIVE = 1, STEP_KERNEL = 2, STEP_OVERFLOW = 4 };

// One Earley byte step at trie depth d (1-based).  The source set is the row's current set for
// d == 1, else the lane's set of depth d-1.  On entry cnt == st.start(d).
template <class S>
__device__ int earley_step(const DeviceTables &T, const uint32_t *__restrict__ bso, const uint2 *__restrict__ bit,
                           uint32_t m, S &st, int d, uint32_t byte, uint32_t &cnt) {
    const uint32_t nb = cnt;
    const uint32_t ncls = T.n_cls, cl = T.cls[byte];
    const uint32_t cur = m - 1 + (uint32_t)(d - 1);   // index of the source set
    const uint32_t SP = (uint32_t)T.N - 1;
    bool ok = true;
    const bool from_base = d == 1;
    uint32_t sb = from_base ? bso[m - 1] : st.start(d - 1);
    uint32_t se = from_base ? bso[m] : nb;
    for (uint32_t i = sb; i < se && ok; i++) {
        uint2 it = from_base ? bit[i] : st.get(i);
        uint32_t p = it.x & 0xFFFFu, q = it.x >> 16;
        uint32_t code = T.sym[p];
        uint32_t k = code >> SYM_KIND_SHIFT;
        if (k == SYM_TERM) {
            uint32_t q2 = T.delta[q * ncls + cl];
            if (q2 == DFA_DEAD) continue;
            uint32_t f = T.qflags[q2];
            if (f & QF_CONT) ok = insert_unique(st, nb, cnt, p | (q2 << 16), it.y);
            if (ok && (f & QF_ACCEPT)) ok = add_advanced(T, st, nb, cnt, p + 1, it.y);
        } else if (k == SYM_NT) {
            uint32_t Y = code & SYM_ID_MASK_NT;
            uint32_t k0 = T.scan_off[Y * ncls + cl], k1 = T.scan_off[Y * ncls + cl + 1];
            for (uint32_t e = k0; e < k1 && ok; e++) {
                uint32_t ent = T.scan_list[e];
                uint32_t p0 = ent & 0xFFFFu, q2 = ent >> 16;
                uint32_t f = T.qflags[q2];
                if (f & QF_CONT) ok = insert_unique(st, nb, cnt, p0 | (q2 << 16), cur);
                if (ok && (f & QF_ACCEPT)) ok = add_advanced(T, st, nb, cnt, p0 + 1, cur);
            }
        }
    }
    bool accepted = false;
    for (uint32_t i = nb; i < cnt && ok; i++) {
        uint2 it = st.get(i);
        uint32_t code = T.sym[it.x & 0xFFFFu];
        if ((code >> SYM_KIND_SHIFT) != SYM_END) continue;
        uint32_t X = code & SYM_ID_MASK;
        if (X == SP) { accepted = true; continue; }
        uint32_t o = it.y;
        const bool in_base = o < m;
        uint32_t jb, je;
        if (in_base) { jb = bso[o]; je = bso[o + 1]; }
        else { int dj = (int)(o - (m - 1)); jb = st.start(dj); je = st.start(dj + 1); }
        for (uint32_t j = jb; j < je && ok; j++) {
            uint2 y = in_base ? bit[j] : st.get(j);
            uint32_t yc = T.sym[y.x & 0xFFFFu];
            if ((yc >> SYM_KIND_SHIFT) != SYM_NT) continue;
            uint32_t Y = yc & SYM_ID_MASK_NT;
            uint32_t c0 = T.comp_off[Y * T.N + X], c1 = T.comp_off[Y * T.N + X + 1];
            for (uint32_t e = c0; e < c1 && ok; e++) ok = add_advanced(T, st, nb, cnt, T.comp_list[e], o);
            if (ok && Y == X) ok = add_advanced(T, st, nb, cnt, (y.x & 0xFFFFu) + 1, y.y);
        }
    }
    if (!ok) return STEP_OVERFLOW;
    const bool alive = cnt > nb || accepted;
    uint32_t w = nb;   // completed items are needed only while their own set is processed
    for (uint32_t i = nb; i < cnt; i++) {
        uint2 it = st.get(i);
        if ((T.sym[it.x & 0xFFFFu] >> SYM_KIND_SHIFT) != SYM_END) { if (w != i) st.put(w, it); w++; }
    }
    cnt = w;
    st.set_start(d + 1, cnt);
    return (alive ? STEP_ALIVE : 0) | (cnt > nb ? STEP_KERNEL : 0);
}

// Walk the nodes of one chunk.  anc(j) gives the node index of the first node's ancestor at
// depth j+1.  Returns false on overflow; otherwise *bits holds the 32 verdicts.
template <class S, class Anc>
__device__ bool walk_chunk(const DeviceTables &T, const uint32_t *bso, const uint2 *bit, uint32_t m, S &st,
                           uint32_t chunk, Anc anc, uint32_t *bits_out) {
    uint32_t i = T.chunk_begin[chunk];
    const uint32_t end = T.chunk_end[chunk];
    const uint32_t rank0 = chunk * CHUNK_RANKS;
    uint32_t bits = 0, cnt = 0;
    st.set_start(1, 0);
    const int d0 = T.nodes[i].depth;
    if (d0 > S::max_depth) return false;
    for (int j = 0; j + 1 < d0; j++) {   // replay the path above the chunk's first node
        TrieNode an = T.nodes[anc(j)];
        int r = earley_step(T, bso, bit, m, st, j + 1, an.byte, cnt);
        if (r & STEP_OVERFLOW) return false;
        if (!(r & STEP_KERNEL)) { i = an.skip; cnt = st.start(j + 1); break; }   // that whole subtree is dead
    }
    while (i < end) {
        TrieNode nd = T.nodes[i];
        int d = nd.depth;
        if (d > S::max_depth) return false;
        cnt = st.start(d);   // forget the sets of the deeper path we came from
        int r = earley_step(T, bso, bit, m, st, d, nd.byte, cnt);
        if (r & STEP_OVERFLOW) return false;
        if (nd.has_string && (r & STEP_ALIVE)) bits |= 1u << (nd.rank - rank0);
        i = (r & STEP_KERNEL) ? i + 1 : nd.skip;
    }
    *bits_out = bits;
    return true;
}

__global__ __launch_bounds__(64) void mask_main_kernel(MaskArgs a) {
    __shared__ uint2 lds_items[LANE_CAP_MAX * 64];
    __shared__ uint8_t lds_ss[(LANE_DEPTH_MAX + 2) * 64];
    const DeviceTables &T = a.tab;
    const uint32_t lane = threadIdx.x, chunk = blockIdx.x * 64 + lane, row = blockIdx.y;
    if (chunk >= (uint32_t)T.n_chunks) return;
    const RowChart rc = a.rows[row];
    const uint32_t *bso = a.set_off + rc.set_base;
    const uint2 *bit = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
    LdsStore st{lds_items + lane, lds_ss + lane, (uint32_t)a.lane_cap};
    const uint32_t *anc_row = T.chunk_anc + (size_t)chunk * CHUNK_ANC;
    uint32_t bits = 0;
    bool ok = walk_chunk(T, bso, bit, rc.n_sets, st, chunk, [&](int j) { return anc_row[j]; }, &bits);
    if (!ok) {
        uint32_t slot = atomicAdd(&a.counters[0], 1u);
        if (slot < a.overflow_cap) a.overflow_list[slot] = make_uint2(row, chunk);
        bits = 0;
    }
    a.rank_mask[(size_t)row * T.Wr + chunk] = bits;
}

// Exact fallback: the same walk, one lane per reported chunk, item list in global memory.
__global__ __launch_bounds__(64) void mask_fallback_kernel(MaskArgs a) {
    const DeviceTables &T = a.tab;
    const uint32_t gid = blockIdx.x * 64 + threadIdx.x;
    uint32_t n = a.counters[0];
    if (n > a.overflow_cap) { if (gid == 0) atomicAdd(&a.counters[1], n - a.overflow_cap); n = a.overflow_cap; }
    GlobalStore st{a.fb_items + gid, a.fb_set_start + gid, (uint32_t)FB_ITEMS_PER_LANE};
    for (uint32_t e = gid; e < n; e += FB_LANES) {
        const uint2 ent = a.overflow_list[e];
        const uint32_t row = ent.x, chunk = ent.y;
        const RowChart rc = a.rows[row];
        const uint32_t *bso = a.set_off + rc.set_base;
        const uint2 *bit = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
        const uint32_t first = T.chunk_begin[chunk];
        const int d0 = T.nodes[first].depth;
        auto anc = [&](int j) {   // ancestor at depth j+1 through the parent links
            uint32_t x = first;
            for (int k = d0; k > j + 1; k--) x = T.parent[x];
            return x;
        };
        uint32_t bits = 0;
        if (!walk_chunk(T, bso, bit, rc.n_sets, st, chunk, anc, &bits)) { atomicAdd(&a.counters[1], 1u); bits = 0; }
        a.rank_mask[(size_t)row * T.Wr + chunk] = bits;
    }
}

// Verdicts are produced in trie order; the caller wants bit v at word v >> 5.  One lane per
// token looks its bit up and a wavefront ballot packs 64 of them into two words.
__global__ __launch_bounds__(256) void permute_kernel(MaskArgs a) {
    const DeviceTables &T = a.tab;
    const uint32_t v = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y;
    uint32_t bit = 0;
    if (v < (uint32_t)T.V) {
        uint32_t r = T.rank_of[v];
        if (r != 0xFFFFFFFFu) bit = (a.rank_mask[(size_t)row * T.Wr + (r >> 5)] >> (r & 31)) & 1u;
    }
    unsigned long long b = __ballot(bit);
    const uint32_t lane = threadIdx.x & 63;
    if ((lane & 31) == 0) {
        uint32_t w = v >> 5;
        if (w < (uint32_t)T.W) a.out_mask[(size_t)row * T.W + w] = (uint32_t)(b >> lane);
    }
}

// Logit masking (Section 3.3): pure copy-or-(-inf).  16-byte accesses, consecutive lanes on
// consecutive 16-byte pieces; the mask words come from L2.
template <typename VecT, int EPV /* elements per 16 bytes */, typename ElemT>
__global__ __launch_bounds__(256) void apply_mask_vec_kernel(const ElemT *__restrict__ in, ElemT *__restrict__ out, int64_t stride,
                                                             int V, int W, const uint32_t *__restrict__ mask, ElemT neg_inf) {
    const int row = blockIdx.y;
    const ElemT *src = in + (size_t)row * stride;
    ElemT *dst = out + (size_t)row * stride;
    const uint32_t *mrow = mask + (size_t)row * W;
    const int n_vec = V / EPV;
    for (int g = blockIdx.x * 256 + threadIdx.x; g < n_vec; g += gridDim.x * 256) {
        VecT x = reinterpret_cast<const VecT *>(src)[g];
        const int v0 = g * EPV;
        const uint32_t mb = mrow[v0 >> 5] >> (v0 & 31);
        ElemT *e = reinterpret_cast<ElemT *>(&x);
#pragma unroll
        for (int k = 0; k < EPV; k++) if (!((mb >> k) & 1u)) e[k] = neg_inf;
        reinterpret_cast<VecT *>(dst)[g] = x;
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

hipError_t launch_mask_main(const MaskArgs &a, hipStream_t s) {
    dim3 grid((a.tab.n_chunks + 63) / 64, a.batch);
    hipLaunchKernelGGL(mask_main_kernel, grid, dim3(64), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_mask_fallback(const MaskArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(mask_fallback_kernel, dim3(FB_LANES / 64), dim3(64), 0, s, a);
    return hipGetLastError();
}
hipError_t launch_permute(const MaskArgs &a, hipStream_t s) {
    dim3 grid((a.tab.V + 255) / 256, a.batch);
    hipLaunchKernelGGL(permute_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_apply_mask(const void *logits, void *out, int dtype, int batch, int64_t row_stride, int V, int W,
                             const uint32_t *mask, hipStream_t s) {
    const size_t esz = dtype == 0 ? 4 : 2;
    const bool aligned = ((uintptr_t)logits % 16 == 0) && ((uintptr_t)out % 16 == 0) && ((row_stride * esz) % 16 == 0);
    const int epv = (int)(16 / esz);
    int blocks_x = aligned ? (V / epv + 255) / 256 : (V + 255) / 256;
    if (blocks_x < 1) blocks_x = 1;
    dim3 grid(blocks_x, batch);
    if (dtype == 0) {
        const uint32_t ninf = 0xFF800000u;
        if (aligned) hipLaunchKernelGGL((apply_mask_vec_kernel<uint4, 4, uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)logits, (uint32_t *)out, row_stride, V, W, mask, ninf);
        else hipLaunchKernelGGL((apply_mask_scalar_kernel<uint32_t>), grid, dim3(256), 0, s, (const uint32_t *)logits, (uint32_t *)out, row_stride, V, W, mask, ninf);
    } else {
        const uint16_t ninf = 0xFF80u;
        if (aligned) hipLaunchKernelGGL((apply_mask_vec_kernel<uint4, 8, uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)logits, (uint16_t *)out, row_stride, V, W, mask, ninf);
        else hipLaunchKernelGGL((apply_mask_scalar_kernel<uint16_t>), grid, dim3(256), 0, s, (const uint16_t *)logits, (uint16_t *)out, row_stride, V, W, mask, ninf);
    }
    return hipGetLastError();
}

}  // namespace zf
