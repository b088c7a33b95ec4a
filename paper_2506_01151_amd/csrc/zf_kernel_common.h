// Device-side pieces shared by the mask kernels: the view of the grammar tables (in LDS or in global
// memory), their staging, one DFA step, and the row's uploaded chart.
#pragma once
#include <hip/hip_runtime.h>
#include "zf_launch.h"

namespace zf {
namespace {

// Table view used by the device code; the pointers lead into LDS or global memory.
struct TV {
    const uint32_t *advpq;
    const uint8_t *cls;
    const uint32_t *qinfo;
    const uint32_t *scan_off;
    const uint32_t *comp_off;
    const uint32_t *delta;
    const uint2 *scan_list;
    const uint32_t *comp_list;
    uint32_t N, ncls, end_base;
};

__device__ __forceinline__ void copy16(void *dst, const void *src, uint32_t bytes, uint32_t tid, uint32_t nthreads) {
    const uint4 *s = reinterpret_cast<const uint4 *>(src);
    uint4 *d = reinterpret_cast<uint4 *>(dst);
    for (uint32_t i = tid; i < bytes / 16; i += nthreads) d[i] = s[i];
}

// Stage the tables the MODE asks for into LDS at smem and build the view.  Returns the bytes used.
// The caller must put a barrier between this and the first use.
template <int MODE>
__device__ __forceinline__ uint32_t stage_tables(const DeviceTables &D, uint8_t *smem, TV &tv, uint32_t tid, uint32_t nthreads) {
    tv.N = D.N; tv.ncls = D.n_cls; tv.end_base = D.end_base;
    uint32_t off = 0;
    if (MODE <= 1) {
        const void *src[5] = {D.advpq, D.cls, D.qinfo, D.scan_off, D.comp_off};
        uint32_t at[5];
#pragma unroll
        for (int k = 0; k < 5; k++) { at[k] = off; copy16(smem + off, src[k], D.small_bytes[k], tid, nthreads); off += D.small_bytes[k]; }
        tv.advpq = reinterpret_cast<const uint32_t *>(smem + at[0]);
        tv.cls = smem + at[1];
        tv.qinfo = reinterpret_cast<const uint32_t *>(smem + at[2]);
        tv.scan_off = reinterpret_cast<const uint32_t *>(smem + at[3]);
        tv.comp_off = reinterpret_cast<const uint32_t *>(smem + at[4]);
    } else {
        tv.advpq = D.advpq; tv.cls = D.cls; tv.qinfo = D.qinfo; tv.scan_off = D.scan_off; tv.comp_off = D.comp_off;
    }
    if (MODE == 0) {
        const void *src[3] = {D.delta, D.scan_list, D.comp_list};
        uint32_t at[3];
#pragma unroll
        for (int k = 0; k < 3; k++) { at[k] = off; copy16(smem + off, src[k], D.big_bytes[k], tid, nthreads); off += D.big_bytes[k]; }
        tv.delta = reinterpret_cast<const uint32_t *>(smem + at[0]);
        tv.scan_list = reinterpret_cast<const uint2 *>(smem + at[1]);
        tv.comp_list = reinterpret_cast<const uint32_t *>(smem + at[2]);
    } else {
        tv.delta = D.delta; tv.scan_list = reinterpret_cast<const uint2 *>(D.scan_list); tv.comp_list = D.comp_list;
    }
    return off;
}

// The same view without the copy: the tables of the MODE are expected at the start of smem in the
// order of DeviceTables::table_blob (the caller copies that prefix).  Returns the bytes they take.
template <int MODE>
__device__ __forceinline__ uint32_t table_view(const DeviceTables &D, uint8_t *smem, TV &tv) {
    tv.N = D.N; tv.ncls = D.n_cls; tv.end_base = D.end_base;
    tv.advpq = D.advpq; tv.cls = D.cls; tv.qinfo = D.qinfo; tv.scan_off = D.scan_off; tv.comp_off = D.comp_off;
    tv.delta = D.delta; tv.scan_list = reinterpret_cast<const uint2 *>(D.scan_list); tv.comp_list = D.comp_list;
    uint32_t off = 0;
    if (MODE <= 1) {
        tv.advpq = reinterpret_cast<const uint32_t *>(smem + off); off += D.small_bytes[0];
        tv.cls = smem + off; off += D.small_bytes[1];
        tv.qinfo = reinterpret_cast<const uint32_t *>(smem + off); off += D.small_bytes[2];
        tv.scan_off = reinterpret_cast<const uint32_t *>(smem + off); off += D.small_bytes[3];
        tv.comp_off = reinterpret_cast<const uint32_t *>(smem + off); off += D.small_bytes[4];
    }
    if (MODE == 0) {
        tv.delta = reinterpret_cast<const uint32_t *>(smem + off); off += D.big_bytes[0];
        tv.scan_list = reinterpret_cast<const uint2 *>(smem + off); off += D.big_bytes[1];
        tv.comp_list = reinterpret_cast<const uint32_t *>(smem + off); off += D.big_bytes[2];
    }
    return off;
}

// One DFA step: returns next state | flags of the next state << 16, or DFA_DEAD in the low half.
__device__ __forceinline__ uint32_t dfa_next(const TV &T, uint32_t q, uint32_t byte, uint32_t cl) {
    const uint32_t info = T.qinfo[q];
    if (info & QF_LITERAL) return (((info >> 8) & 0xFFu) == byte && (info & QF_CONT)) ? ((q + 1) | (info & 0xFFFF0000u)) : (uint32_t)DFA_DEAD;
    return T.delta[(info >> 16) * T.ncls + cl];
}

template <class SoPtr, class ItPtr>
struct Base {                  // the row's uploaded chart (LDS copy or global)
    SoPtr so;                  // set offsets, so[k] .. so[k+1]
    ItPtr it;                  // items: x = item word, y = origin
    uint32_t m;                // number of sets; set m-1 is the current one
    uint32_t last_lo, last_hi; // so[m-1], so[m]
};
typedef Base<const uint32_t *, const uint2 *> BaseG;

__device__ __forceinline__ BaseG global_base(const MaskArgs &a, uint32_t row) {
    const RowChart rc = a.rows[row];
    BaseG B;
    B.so = a.set_off + rc.set_base;
    B.it = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
    B.m = rc.n_sets;
    B.last_lo = B.so[rc.n_sets - 1];
    B.last_hi = B.so[rc.n_sets];
    return B;
}

// What the last kernel of a call does at the end of every block: one block copies the call's counters to pinned host memory,
// clears the next call's set, and then writes the word the host polls.  ticketed = false: the counters were final before this
// kernel started (nothing in it can fail), and the block with the highest index does it at its end: the word then says "the
// status is known", and readers of the mask are ordered behind the kernel by the stream.  ticketed = true (the closing kernel
// with a fallback pass to run, whose waits can fail): every block draws a ticket when it is done and the block that draws
// the last one does it, so that no error is counted after the hand-over.  Tickets are drawn in two levels (group of blocks,
// then groups); even so they cost the kernel 5 us at 2,004 blocks (a ticket is a round trip to memory), which is why the
// common case does without.  (An error count is a device-scope atomic followed by the counting wavefront's own release
// fence; a fence in every block would write the L2 back each time: 6 -> 34 us.)
__device__ __forceinline__ void hand_over(const MaskArgs &a, uint32_t lin, uint32_t n_blocks, bool ticketed, uint32_t block_sum = 0, bool count_only = false) {
    __shared__ uint32_t last;
    unsigned long long *tickets = reinterpret_cast<unsigned long long *>(a.counters + TICKET_AT);
    const uint32_t n_groups = n_blocks < (uint32_t)TICKET_GROUPS ? n_blocks : (uint32_t)TICKET_GROUPS;
    if (count_only) {                                        // not the call's last kernel: leave the block's share of counter [1] only
        if (threadIdx.x == 0 && block_sum) atomicAdd(&tickets[lin % n_groups], (unsigned long long)block_sum << 32);
        return;
    }
    if (!ticketed) { if (lin != n_blocks - 1) return; }
    __syncthreads();
    if (ticketed) {
        if (threadIdx.x == 0) {
            const uint32_t g = lin % n_groups, size = n_blocks / n_groups + (g < n_blocks % n_groups ? 1u : 0u);
            uint32_t is_last = 0;
            if ((uint32_t)atomicAdd(&tickets[g], ((unsigned long long)block_sum << 32) | 1ull) == size - 1) is_last = atomicAdd(&a.counters[TICKET_TOP], 1u) == n_groups - 1 ? 1u : 0u;
            last = is_last;
        }
        __syncthreads();
        if (!last) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    uint32_t part = 0, x = 0;
    const uint32_t k = threadIdx.x;
    if (k < 64) {                                            // the counters, one per lane (their loads travel together), and the partial sums of counter [1]
        part = (uint32_t)(__hip_atomic_load(&tickets[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d);
        if (k < 4) x = __hip_atomic_load(&a.counters[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else if (k >= 5 && k < 8 && a.store.ctl) x = __hip_atomic_load(&a.store.ctl[k - 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (k == 1) x += part;
    }
    // persistent automaton: where every row of the call stands now (the first round of these loads travels with the counters')
    uint32_t row0 = 0;
    if (a.store_row_dev && k < (uint32_t)a.batch) row0 = __hip_atomic_load(&a.store_row_dev[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();                                         // the ticket words have been read: now the next call's set is cleared (it may be this very set's neighbour only, never this set)
    for (uint32_t i = threadIdx.x; i < (uint32_t)COUNTER_SET_WORDS; i += blockDim.x) a.counters_next[i] = 0;   // the next call's set (no separate memset)
    if (a.store_row_dev) {
        if (k < (uint32_t)a.batch) a.store_row_out[k] = row0;
        for (uint32_t i = k + blockDim.x; i < (uint32_t)a.batch; i += blockDim.x) a.store_row_out[i] = __hip_atomic_load(&a.store_row_dev[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();                                         // ... before the first wavefront's release below
    if (k < 64) {                                            // counters first, then the word the host waits for
        if (k < 4 || (k >= 5 && k < 8 && a.store.ctl)) a.host_status[k] = x;
        if (k == 0) __hip_atomic_store(&a.host_status[4], a.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);   // a release of the wavefront's stores
    }
}

inline uint32_t table_bytes(const DeviceTables &t, int mode) {
    uint32_t n = 0;
    if (mode <= 1) for (int k = 0; k < 5; k++) n += t.small_bytes[k];
    if (mode == 0) for (int k = 0; k < 3; k++) n += t.big_bytes[k];
    return n;
}

}  // namespace
}  // namespace zf
