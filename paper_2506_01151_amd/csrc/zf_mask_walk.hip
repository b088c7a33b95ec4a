// Mask kernels, trie walk: cache_merge_kernel + mask_walk_kernel (zf_options.walk_mode = 1) and
// finish_kernel (the exact fallback pass of both mask kernels + the permutation into token order).
//
// The vocabulary trie is stored in preorder, so a depth-first walk is a linear scan in which a
// dead subtree is left through the node's skip pointer and a shared prefix is scanned once.  A
// chunk is the node range of `chunk_ranks` consecutive strings; the merge kernel applies the
// context-independent token-mask cache (Section 4.3) and queues the chunks that hold undecided
// strings, and a persistent grid of wavefronts walks them, one Earley byte step (Scan + Complete
// with tabulated Predict, Section 3.2) per live trie node, on an item list in LDS that holds one
// set per trie depth of the current path.  The step is wavefront-cooperative with uniform control
// flow (wave_step): items of a set are spread over the lanes, the set under construction is held
// in registers, duplicate tests are ballots.  (Giving every lane its own chunk was measured first:
// the nests of short data-dependent loops of an Earley step then cost ~12,000 cycles per step per
// wavefront because every loop level runs for its longest trip count over the 64 lanes.)  Grammar
// tables are staged in LDS once per block.  What does not fit the LDS budgets repeats the walk in
// the fallback pass (part of finish_kernel), one wavefront per chunk, with the item list in a global-memory arena.
#include "zf_kernel_common.h"
#include "zf_aut_step.h"

namespace zf {
namespace {

// ---- item-list storage policies ---------------------------------------------------------
// An item is (w, o): w = item word (see IW_* in zf_device.h), o = origin set.
struct WaveLdsStore {          // walk kernel: the wavefront's list in LDS; set starts in a register (lane d holds the start of depth d)
    uint32_t *pq;
    uint32_t *org;
    uint32_t ss_reg;
    uint32_t lane;
    uint32_t cap;
    static constexpr int max_depth = WALK_DEPTH_MAX;
    __device__ __forceinline__ void get(uint32_t i, uint32_t &p, uint32_t &o) const { p = pq[i]; o = org[i]; }
    __device__ __forceinline__ void put(uint32_t i, uint32_t p, uint32_t o) { pq[i] = p; org[i] = o; }
    __device__ __forceinline__ uint32_t start(int d) const { return (uint32_t)__builtin_amdgcn_readlane((int)ss_reg, __builtin_amdgcn_readfirstlane(d)); }
    __device__ __forceinline__ void set_start(int d, uint32_t v) { if ((int)lane == d) ss_reg = v; }
};
struct GlobalStore {           // fallback: the wavefront's list in a global-memory arena
    uint2 *items;
    uint32_t *ss;
    uint32_t cap;
    static constexpr int max_depth = FB_DEPTH_MAX;
    __device__ __forceinline__ void get(uint32_t i, uint32_t &p, uint32_t &o) const { const uint2 x = items[i]; p = x.x; o = x.y; }
    __device__ __forceinline__ void put(uint32_t i, uint32_t p, uint32_t o) { items[i] = make_uint2(p, o); }
    __device__ __forceinline__ uint32_t start(int d) const { return ss[d]; }
    __device__ __forceinline__ void set_start(int d, uint32_t v) { ss[d] = v; }
};

enum { STEP_ALIVE = 1, STEP_KERNEL = 2, STEP_OVERFLOW = 4, STEP_WIDE = 8 /* a set wider than 64 items: redo with wave_step_big */ };

// One Earley byte step at trie depth d (1-based): the narrow variant of the shared wavefront-cooperative step
// (zf_aut_step.h), with the wavefront's item list as the sets view.  The source set is the row's current set for
// d == 1, else the wavefront's set of depth d-1.  On entry cnt == st.start(d); on exit the new set is stored at
// [cnt_in, cnt_out).  All 64 lanes call it with identical arguments.  A new set of more than 64 items is reported
// as STEP_WIDE (wave_step_big takes it), an exhausted item budget as STEP_OVERFLOW (the fallback pass takes the chunk).
template <class BaseT>
struct WalkSets {              // a set named by its index: a set of the row's chart, or the wavefront's set of one trie depth
    const BaseT B;             // copies: the view is made anew for every step
    const WaveLdsStore st;
    static constexpr uint64_t IN_LIST = 1ull << 32;   // handle: index of the set's first item, in the wavefront's list with this bit, else in the row's chart
    __device__ __forceinline__ void view(uint32_t ref, uint64_t &h, uint32_t &n) const {
        if (ref + 1 == B.m) { h = B.last_lo; n = B.last_hi - B.last_lo; }   // the row's current set: its bounds are at hand, no load
        else if (ref < B.m) { const uint32_t lo = B.so[ref]; h = lo; n = B.so[ref + 1] - lo; }
        else { const int dj = (int)(ref - (B.m - 1)); const uint32_t lo = st.start(dj); h = IN_LIST | lo; n = st.start(dj + 1) - lo; }
    }
    __device__ __forceinline__ uint2 item(uint64_t h, uint32_t i) const {
        const uint32_t k = (uint32_t)h + i;
        if (h & IN_LIST) return make_uint2(st.pq[k], st.org[k]);
        return B.it[k];
    }
};
template <class BaseT>
__device__ __forceinline__ int wave_step(const TV &T, const BaseT &B, WaveLdsStore &st, int d, uint32_t byte, uint32_t cl, uint32_t &cnt, uint32_t lane) {
    const uint32_t nb = cnt;                             // nb <= cap always
    const WalkSets<BaseT> S{B, st};
    uint32_t nnew = 0, kept = 0;
    const int r = aut_step_narrow<false, true>(T, S, st.pq + nb, st.org + nb, st.cap - nb, B.m - 1 + (uint32_t)(d - 1), byte, cl, lane, nnew, kept);
    if (r == AUT_WIDE) return STEP_WIDE;
    if (r == AUT_OVER) return STEP_OVERFLOW;
    cnt = nb + kept;
    st.set_start(d + 1, cnt);
    return (nnew ? STEP_ALIVE : 0) | (kept ? STEP_KERNEL : 0);
}

// The wavefront step for large sets (ambiguous grammars make sets of hundreds of items): same
// structure, but the set under construction lives in LDS only and every loop over items runs in
// strips of 64.  Slower per item than wave_step, used only when a set does not fit 64 lanes.
template <class BaseT, class S>
__device__ __forceinline__ int wave_step_big(const TV &T, const BaseT &B, S &st, int d, uint32_t byte, uint32_t cl, uint32_t &cnt, uint32_t lane) {
    const uint32_t nb = cnt;
    const uint32_t cur = B.m - 1 + (uint32_t)(d - 1);
    const bool from_base = d == 1;
    const uint32_t sb = from_base ? B.last_lo : st.start(d - 1);
    const uint32_t se = from_base ? B.last_hi : nb;
    uint32_t nnew = 0;
    bool saw_end = false, failed = false;                // failed: the item budget is used up (sticky; the step runs on and reports at its end)
    auto insert = [&](uint32_t w, uint32_t o) {
        unsigned long long dup = 0;
        for (uint32_t s0 = 0; s0 < nnew; s0 += 64) {
            uint32_t xw = 0, xo = 0xFFFFFFFFu;
            if (s0 + lane < nnew) st.get(nb + s0 + lane, xw, xo);
            dup |= __ballot(s0 + lane < nnew && xw == w && xo == o);
        }
        const bool add = !dup && nb + nnew < st.cap;
        failed |= !dup && !add;
        if (add && lane == 0) st.put(nb + nnew, w, o);
        nnew += add ? 1u : 0u;
    };
    auto advance = [&](uint32_t p, uint32_t o) {
        for (;;) {
            const uint32_t w = T.advpq[p];
            insert(w, o);
            if (w & IW_END) { saw_end = true; return; }
            if ((w & IW_TERM) || !(w & IW_NT_NULLABLE)) return;
            p++;
        }
    };
    for (uint32_t s0 = sb; s0 < se; s0 += 64) {
        uint32_t sw = IW_END, so = 0;
        if (s0 + lane < se) { if (from_base) { const uint2 x = B.it[s0 + lane]; sw = x.x; so = x.y; } else st.get(s0 + lane, sw, so); }
        uint32_t nx = DFA_DEAD;
        if (sw & IW_TERM) nx = dfa_next(T, sw >> 16, byte, cl);
        unsigned long long m = __ballot((nx & 0xFFFFu) != DFA_DEAD);
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t lw = __builtin_amdgcn_readlane(sw, l), lo = __builtin_amdgcn_readlane(so, l), lnx = __builtin_amdgcn_readlane(nx, l);
            if ((lnx >> 16) & QF_CONT) insert((lw & 0xFFFFu) | (lnx << 16), lo);
            if ((lnx >> 16) & QF_ACCEPT) advance((lw & IW_POS_MASK) + 1, lo);
        }
        m = __ballot(!(sw & (IW_TERM | IW_END)));
        while (m) {
            const int l = __ffsll((long long)m) - 1;
            m &= m - 1;
            const uint32_t Y = (__builtin_amdgcn_readlane(sw, l) >> IW_NT_SHIFT) & IW_NT_MASK;
            const uint32_t k0 = T.scan_off[Y * T.ncls + cl], k1 = T.scan_off[Y * T.ncls + cl + 1];
            for (uint32_t e = k0; e < k1; e++) {
                const uint2 ef = T.scan_list[e];
                if (ef.y & QF_CONT) insert(ef.x, cur);
                if (ef.y & QF_ACCEPT) advance((ef.x & IW_POS_MASK) + 1, cur);
            }
        }
    }
    if (saw_end) {
        for (uint32_t i = 0; i < nnew; i++) {
            uint32_t w, o;
            st.get(nb + i, w, o);                        // every lane reads the same item
            if (!(w & IW_END)) continue;
            const uint32_t X = (w & IW_POS_MASK) - T.end_base;
            if (X == T.N - 1) continue;
            const bool in_base = o < B.m;
            uint32_t jb, je;
            if (in_base) { jb = B.so[o]; je = B.so[o + 1]; }
            else { const int dj = (int)(o - (B.m - 1)); jb = st.start(dj); je = st.start(dj + 1); }
            for (uint32_t j0 = jb; j0 < je; j0 += 64) {
                uint32_t yw = IW_END, yo = 0;
                if (j0 + lane < je) { if (in_base) { const uint2 y = B.it[j0 + lane]; yw = y.x; yo = y.y; } else st.get(j0 + lane, yw, yo); }
                const bool nt = !(yw & (IW_TERM | IW_END));
                const uint32_t Y = (yw >> IW_NT_SHIFT) & IW_NT_MASK;
                uint32_t c0 = 0, c1 = 0;
                if (nt) { c0 = T.comp_off[Y * T.N + X]; c1 = T.comp_off[Y * T.N + X + 1]; }
                unsigned long long mm = __ballot(nt && c1 > c0);
                while (mm) {
                    const int l = __ffsll((long long)mm) - 1;
                    mm &= mm - 1;
                    const uint32_t lc0 = __builtin_amdgcn_readlane(c0, l), lc1 = __builtin_amdgcn_readlane(c1, l);
                    for (uint32_t e = lc0; e < lc1; e++) {
                        const uint32_t cw = T.comp_list[e];
                        if (cw != 0xFFFFFFFFu) insert(cw, o);
                        else advance((__builtin_amdgcn_readlane(yw, l) & IW_POS_MASK) + 1, __builtin_amdgcn_readlane(yo, l));
                    }
                }
            }
        }
    }
    if (failed) return STEP_OVERFLOW;
    // drop the completed items: forward compaction, strip by strip (a strip is read before it is written)
    uint32_t kept = 0;
    for (uint32_t s0 = 0; s0 < nnew; s0 += 64) {
        uint32_t w = IW_END, o = 0;
        if (s0 + lane < nnew) st.get(nb + s0 + lane, w, o);
        const bool keep = !(w & IW_END);
        const unsigned long long kb = __ballot(keep);
        if (keep) st.put(nb + kept + __popcll(kb & ((1ull << lane) - 1ull)), w, o);
        kept += (uint32_t)__popcll(kb);
    }
    cnt = nb + kept;
    st.set_start(d + 1, cnt);
    return (nnew ? STEP_ALIVE : 0) | (kept ? STEP_KERNEL : 0);
}

// What a wavefront remembers between two chunks of the same row: which trie path its stored sets
// belong to.  A node is named by (depth, rank of its first string).  Consecutive chunks share most
// of the path above their first node, so the next walk replays only what differs.
struct PathMemo {
    uint32_t rank_at;          // lane d: the node whose live set is stored at depth d (valid for 1 <= d <= valid)
    int valid;                 // depths 1..valid hold live sets of one root path
    int dead_depth;            // the node (dead_depth, dead_rank) below that path is known to leave no item: its subtree is dead
    uint32_t dead_rank;
    __device__ __forceinline__ void reset() { rank_at = 0; valid = 0; dead_depth = 0; dead_rank = 0; }
    __device__ __forceinline__ void note(int d, uint32_t rank, bool live, uint32_t lane) {   // a step was taken at depth d
        if (live) { valid = d; dead_depth = 0; if ((int)lane == d) rank_at = rank; }
        else { valid = d - 1; dead_depth = d; dead_rank = rank; }
    }
};

// Walk the nodes of one chunk.  anc(j) gives the first node's ancestor at depth j+1.  Returns
// false on overflow (the memo is then unusable); otherwise *bits_out holds the chunk's verdicts.
// `want` marks the strings of the chunk that still need a verdict (the others are decided by the
// token-mask cache); subtrees without such a string are skipped without a byte step.
template <class S, class Step, class Anc, class Nodes>
__device__ __forceinline__ bool walk_chunk(const DeviceTables &D, S &st, Step step, uint32_t chunk, uint32_t want,
                                           uint32_t begin, uint32_t end, Anc anc, Nodes node, uint32_t *bits_out,
                                           PathMemo &memo, uint32_t lane) {
    uint32_t i = begin;
    const uint32_t rank0 = chunk * (uint32_t)D.chunk_ranks;
    uint32_t bits = 0, cnt = 0;
    st.set_start(1, 0);
    TrieNode nd = node(i);
    const int n_anc = nd.depth - 1;                      // the path above the chunk's first node: reused or replayed
    if (nd.depth > S::max_depth) return false;
    int j = 0;
    while (j < n_anc && j < memo.valid && (uint32_t)__builtin_amdgcn_readlane((int)memo.rank_at, j + 1) == anc(j).rank) j++;
    if (j < n_anc && memo.dead_depth == j + 1 && j == memo.valid) {
        const TrieNode dn = anc(j);
        if (dn.rank == memo.dead_rank) {                 // the chunk starts inside a subtree known to be dead
            i = dn.skip; j = n_anc;
            if (i < end) nd = node(i);
        }
    } else if (j < memo.valid) { memo.valid = j; memo.dead_depth = 0; }
    cnt = st.start(j + 1);
    for (;;) {                                           // one loop, one call site of the byte step (keeps the code small)
        const bool warm = j < n_anc;
        const uint32_t nxt = i + 1;
        TrieNode cur, nx = nd;
        uint32_t rel = 0;
        bool do_step = true;
        if (warm) cur = anc(j);
        else {
            if (i >= end) break;
            cur = nd;
            if (nxt < end) nx = node(nxt);               // issued before the step so that it overlaps it
            rel = cur.rank - rank0;
            const uint32_t span = (cur.n_sub >= 32u ? 0xFFFFFFFFu : ((1u << cur.n_sub) - 1u)) << rel;
            do_step = (span & want) != 0;                // nothing to decide below this node: skip it without a step
            if (do_step) {
                if (cur.depth > S::max_depth) return false;
                cnt = st.start(cur.depth);               // forget the sets of the deeper path we came from
            }
        }
        int r = 0;
        if (do_step) {
            const int d = warm ? j + 1 : (int)cur.depth;
            r = step(d, cur.byte, cur.cls, cnt);
            if (r & STEP_OVERFLOW) return false;
            memo.note(d, cur.rank, (r & STEP_KERNEL) != 0, lane);
        }
        if (warm) {
            if (r & STEP_KERNEL) { j++; continue; }
            i = cur.skip; cnt = st.start(j + 1); j = n_anc;   // that whole subtree is dead
            if (i < end) nd = node(i);
            continue;
        }
        if (cur.has_string && (r & STEP_ALIVE)) bits |= 1u << rel;
        const uint32_t ni = (r & STEP_KERNEL) ? nxt : cur.skip;
        if (ni == nxt) nd = nx;
        else if (ni < end) nd = node(ni);
        i = ni;
    }
    *bits_out = bits;
    return true;
}

__device__ __forceinline__ uint32_t load_bits(const DeviceTables &D, const uint32_t *bitmap_row, uint32_t chunk) {
    const uint8_t *rowp = reinterpret_cast<const uint8_t *>(bitmap_row);
    if (D.chunk_ranks == 32) return reinterpret_cast<const uint32_t *>(rowp)[chunk];
    if (D.chunk_ranks == 16) return reinterpret_cast<const uint16_t *>(rowp)[chunk];
    return rowp[chunk];
}

__device__ __forceinline__ void store_bits(const DeviceTables &D, uint32_t *rank_mask, uint32_t row, uint32_t chunk, uint32_t bits) {
    uint8_t *rowp = reinterpret_cast<uint8_t *>(rank_mask + (size_t)row * D.Wr);
    if (D.chunk_ranks == 32) reinterpret_cast<uint32_t *>(rowp)[chunk] = bits;
    else if (D.chunk_ranks == 16) reinterpret_cast<uint16_t *>(rowp)[chunk] = (uint16_t)bits;
    else rowp[chunk] = (uint8_t)bits;
}
// several walks may add verdicts to the same word of the rank-ordered bitmap: atomic OR
__device__ __forceinline__ void or_bits(const DeviceTables &D, uint32_t *rank_mask, uint32_t row, uint32_t chunk, uint32_t bits) {
    if (!bits) return;
    const uint32_t byte_off = chunk * ((uint32_t)D.chunk_ranks >> 3);
    atomicOr(rank_mask + (size_t)row * D.Wr + (byte_off >> 2), bits << ((byte_off & 3u) * 8u));
}

// Token-mask cache (Section 4.3): merge the cached bitsets of every item of the row's current set,
// store the strings some terminal swallows whole, and queue the chunks that hold strings which
// need the parser.  One lane per 64 ranks (two words of the rank-ordered bitmap, 64 / chunk_ranks
// chunks); a wavefront appends its chunks to the queue in chunk order with one atomic, so that
// neighbours in the queue are mostly neighbours in the trie (the walk reuses shared paths).
__global__ __launch_bounds__(256) void cache_merge_kernel(MaskArgs a) {
    const DeviceTables &D = a.tab;
    const uint32_t t = blockIdx.x * 256 + threadIdx.x, row = blockIdx.y, lane = threadIdx.x & 63;
    const RowChart rc = a.rows[row];
    const uint32_t w0 = 2 * t, Wr = (uint32_t)D.Wr, cr = (uint32_t)D.chunk_ranks;
    const bool has0 = w0 < Wr, has1 = w0 + 1 < Wr;
    uint32_t v0 = 0, v1 = 0, c0 = 0, c1 = 0;
    if (has0) {
        if (rc.n_ent == 0) { c0 = 0xFFFFFFFFu; c1 = has1 ? 0xFFFFFFFFu : 0u; }
        for (uint32_t k = 0; k < rc.n_ent; k++) {
            const size_t r = (size_t)a.entries[rc.ent_base + k] * Wr + w0;
            v0 |= D.ci_valid[r]; c0 |= D.ci_cd[r];
            if (has1) { v1 |= D.ci_valid[r + 1]; c1 |= D.ci_cd[r + 1]; }
        }
        a.rank_mask[(size_t)row * Wr + w0] = v0;
        if (has1) a.rank_mask[(size_t)row * Wr + w0 + 1] = v1;
    }
    const unsigned long long want = ((unsigned long long)(c1 & ~v1) << 32) | (c0 & ~v0);
    const uint32_t per_lane = 64u / cr, chunk0 = t * per_lane;
    const unsigned long long cm = cr == 32 ? 0xFFFFFFFFull : ((1ull << cr) - 1ull);
    uint32_t n_mine = 0;
    for (uint32_t k = 0; k < per_lane; k++) n_mine += ((want >> (k * cr)) & cm) != 0 && chunk0 + k < (uint32_t)D.n_chunks;
    if (!__ballot(n_mine != 0)) return;
    uint32_t incl = n_mine;                                  // inclusive prefix sum over the lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) { const uint32_t up = __shfl_up(incl, d); if ((int)lane >= d) incl += up; }
    uint32_t base = 0;
    if (lane == 63) base = atomicAdd(&a.counters[1], incl);
    base = __shfl(base, 63);
    uint32_t at = base + incl - n_mine;
    for (uint32_t k = 0; k < per_lane; k++) {
        const uint32_t wk = (uint32_t)((want >> (k * cr)) & cm), chunk = chunk0 + k;
        if (!wk || chunk >= (uint32_t)D.n_chunks) continue;
        const uint32_t begin = D.chunk_begin[chunk], n_nodes = D.chunk_end[chunk] - begin;
        a.work[at++] = make_uint4(row | (n_nodes > 0xFFFFu ? 0xFFFF0000u : n_nodes << 16), chunk, wk, begin);
    }
}

static const uint32_t BASE_LDS_BYTES = (BASE_SETS_LDS + 1) * 4 + BASE_ITEMS_LDS * 8;
__host__ __device__ inline uint32_t wave_region_bytes(uint32_t cap) {
    // prefetched nodes, ancestor nodes, the row's chart, item words, origins; a multiple of 16
    return (WALK_NODES_LDS + CHUNK_ANC) * 16 + BASE_LDS_BYTES + (cap * 8 + 15) / 16 * 16;
}

struct ParentAnc {             // ancestor node at depth j+1 through the parent links
    const TrieNode *nodes; const uint32_t *parent; uint32_t first; int d0;
    __device__ __forceinline__ TrieNode operator()(int j) const {
        uint32_t x = first;
        for (int k = d0; k > j + 1; k--) x = parent[x];
        return nodes[x];
    }
};

// The parser walk.  Persistent blocks; every wavefront takes queued chunks g, g + stride, ...
template <int MODE>
__global__ __launch_bounds__(WALK_BLOCK) __attribute__((amdgpu_waves_per_eu(6))) void mask_walk_kernel(MaskArgs a) {
    extern __shared__ __align__(16) uint8_t smem[];
    const DeviceTables &D = a.tab;
    const uint32_t tid = threadIdx.x;
    const uint32_t n_work = a.counters[1];
    // The queue is dealt to the blocks in tiles, round robin; a tile is WALK_WAVES runs of `run`
    // consecutive items, and inside a block the wavefronts take the next run of the block's share
    // whenever they are free (LDS counter), so that one long walk does not hold up the items behind
    // it.  Items of a run are mostly neighbouring chunks of one row: the wavefront keeps its path
    // (PathMemo) from one to the next.  Short queues are dealt item by item so that all wavefronts work.
    uint32_t run = n_work / (gridDim.x * WALK_WAVES);
    run = run < 1 ? 1 : (run > WALK_RUN_MAX ? WALK_RUN_MAX : run);
    const uint32_t tile = run * WALK_WAVES;
    if (blockIdx.x * tile >= n_work) return;            // uniform: not even the block's first tile exists
    TV T;
    uint32_t off = stage_tables<MODE>(D, smem, T, tid, WALK_BLOCK);
    uint32_t *next_item = reinterpret_cast<uint32_t *>(smem + off);   // the block's counter of items handed out
    off += 16;
    if (tid == 0) *next_item = 0;
    __syncthreads();                                     // the only block-wide barrier; below, wavefronts run on their own
    const uint32_t wave = tid >> 6, lane = tid & 63;
    const uint32_t cap = (uint32_t)a.lane_cap;
    uint8_t *region = smem + off + wave * wave_region_bytes(cap);
    TrieNode *l_nodes = reinterpret_cast<TrieNode *>(region);
    TrieNode *l_anc = l_nodes + WALK_NODES_LDS;
    uint32_t *l_so = reinterpret_cast<uint32_t *>(region + (WALK_NODES_LDS + CHUNK_ANC) * 16);
    uint2 *l_it = reinterpret_cast<uint2 *>(l_so + BASE_SETS_LDS + 1);
    WaveLdsStore st;
    st.pq = reinterpret_cast<uint32_t *>(l_it + BASE_ITEMS_LDS);
    st.org = st.pq + cap;
    st.ss_reg = 0;
    st.lane = lane;
    st.cap = cap;
    PathMemo memo;
    memo.reset();
    uint32_t memo_row = 0xFFFFFFFFu;
    for (;;) {
        uint32_t k = 0;
        if (lane == 0) k = atomicAdd(next_item, 1u);
        k = (uint32_t)__builtin_amdgcn_readfirstlane((int)k);
        const uint32_t t_base = ((k / WALK_WAVES) * gridDim.x + blockIdx.x) * tile;
        if (t_base >= n_work) break;                    // this and every later tile of this block lie beyond the queue
        const uint32_t g0 = t_base + (k % WALK_WAVES) * run;
        for (uint32_t g = g0; g < g0 + run && g < n_work; g++) {
            const uint4 item = a.work[g];               // row | node count << 16, chunk, undecided strings, first node
            const uint32_t row = item.x & 0xFFFFu, n_nodes = item.x >> 16, chunk = item.y, want = item.z, begin = item.w;
            const RowChart rc = a.rows[row];
            const uint32_t *g_so = a.set_off + rc.set_base;
            const uint2 *g_it = reinterpret_cast<const uint2 *>(a.items) + rc.item_base;
            const bool base_fits = rc.n_sets <= BASE_SETS_LDS && rc.n_items <= BASE_ITEMS_LDS;
            // all 64 lanes pull the chunk's nodes, the ancestors of its first node and the row's chart into LDS
            if (n_nodes <= (uint32_t)WALK_NODES_LDS)
                for (uint32_t k2 = lane; k2 < n_nodes; k2 += 64) l_nodes[k2] = D.nodes[begin + k2];
            if (lane < CHUNK_ANC) l_anc[lane] = D.chunk_anc[(size_t)chunk * CHUNK_ANC + lane];
            if (row != memo_row) {                       // another row: its chart, and no path to reuse
                memo.reset();
                memo_row = row;
                if (base_fits) {
                    for (uint32_t k2 = lane; k2 <= rc.n_sets; k2 += 64) l_so[k2] = g_so[k2];
                    for (uint32_t k2 = lane; k2 < rc.n_items; k2 += 64) l_it[k2] = g_it[k2];
                }
            }
            // lanes read what other lanes of their own wavefront wrote: LDS serves one wavefront's
            // accesses in issue order; the fences keep the compiler from moving accesses across
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            {
                uint32_t bits = 0;
                bool ok = cap > 0 && n_nodes <= (uint32_t)WALK_NODES_LDS && l_nodes[0].depth - 1 <= CHUNK_ANC;
                if (ok) {
                    auto anc = [&](int j) { return l_anc[j]; };
                    auto node = [&](uint32_t i) { return l_nodes[i - begin]; };
                    // the row's chart through generic pointers: its LDS copy when it was staged, else global memory
                    const uint32_t *b_so = base_fits ? l_so : g_so;
                    const uint2 *b_it = base_fits ? l_it : g_it;
                    const BaseG B{b_so, b_it, rc.n_sets, b_so[rc.n_sets - 1], rc.n_items};
                    ok = walk_chunk(D, st, [&](int d, uint32_t byte, uint32_t cl, uint32_t &cnt) {
                                            const uint32_t keep = cnt;
                                            int r = wave_step(T, B, st, d, byte, cl, cnt, lane);
                                            if (r & STEP_WIDE) { cnt = keep; r = wave_step_big(T, B, st, d, byte, cl, cnt, lane); }
                                            return r; },
                                    chunk, want, begin, begin + n_nodes, anc, node, &bits, memo, lane);
                }
                if (!ok) memo.reset();
                if (lane == 0) {
                    if (!ok) {
                        const uint32_t slot = atomicAdd(&a.counters[0], 1u);
                        if (slot < a.overflow_cap) a.overflow_list[slot] = make_uint4(row, chunk, want, 0);
                    } else or_bits(D, a.rank_mask, row, chunk, bits & want);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the next round overwrites the staged data
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// Fallback: one wavefront per chunk that outgrew LDS; same walk with the strip-wise step and the
// item list in a global-memory arena.  Wavefront gw of n_waves takes entries gw, gw + n_waves, ... of the
// n listed ones.
__device__ __forceinline__ void fallback_wave(const MaskArgs &a, uint32_t gw, uint32_t n_waves, uint32_t n, uint32_t lane) {
    const DeviceTables &D = a.tab;
    TV T;
    stage_tables<2>(D, nullptr, T, 0, 1);
    if (n > a.overflow_cap) { if (gw == 0 && lane == 0) atomicAdd(&a.counters[2], n - a.overflow_cap); n = a.overflow_cap; }
    GlobalStore st{a.fb_items + (size_t)gw * a.fb_stride, a.fb_set_start + (size_t)gw * (FB_DEPTH_MAX + 2), (uint32_t)a.fb_cap};
    for (uint32_t e = gw; e < n; e += n_waves) {
        const uint4 ent = a.overflow_list[e];
        const BaseG B = global_base(a, ent.x);
        const uint32_t begin = D.chunk_begin[ent.y], end = D.chunk_end[ent.y];
        ParentAnc anc{D.nodes, D.parent, begin, D.nodes[begin].depth};
        uint32_t bits = 0;
        PathMemo memo;
        memo.reset();
        const bool ok = walk_chunk(D, st, [&](int d, uint32_t byte, uint32_t cl, uint32_t &cnt) { return wave_step_big(T, B, st, d, byte, cl, cnt, lane); },
                                   ent.y, ent.z, begin, end, anc, [&](uint32_t i) { return D.nodes[i]; }, &bits, memo, lane);
        if (lane == 0) {
            if (!ok) atomicAdd(&a.counters[2], 1u);
            else or_bits(D, a.rank_mask, ent.x, ent.y, bits & ent.z);
        }
        // lanes write the arena, lane-uniform reads follow in the next round: keep the order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// The closing kernel of a call: the fallback pass (rare) and the permutation of the verdicts from
// string-rank order into token order, in one launch.  As a kernel of its own the fallback pass costs
// 4.5 us per call even when its list is empty (a launch and two dependent loads), and with the mask
// automata almost every call leaves it empty.
//   When the list is not empty, the wavefronts of the blocks with the lowest linear index walk the
// listed chunks first and count themselves off; every block then waits for that count before it
// reads the verdicts.  The host sizes the grid so that the chip holds all of its blocks at once
// (blocks loop over row groups when a batch has more of them): every block that waits is resident
// together with the wavefronts it waits for, whatever the order the blocks were started in, and the
// fallback wavefronts wait for nothing, so the wait ends.  It is bounded all the same, and running
// into the bound makes the call fail with ZF_ERR_OVERFLOW.
//   Permutation: verdicts are produced in trie order, the caller wants bit v at word v >> 5.  One lane
// per token and PERMUTE_ROWS rows looks the token's rank up once, and a wavefront ballot packs 64
// verdicts into two words.
//   Hand-over: see hand_over (zf_kernel_common.h).
static const int FINISH_BLOCK = 256;
static const int FINISH_WAVES = FINISH_BLOCK / 64;
static const int PERMUTE_ROWS = 4;
static const int PERMUTE_AHEAD = 4;                   // rank look-ups a thread has in flight
static const uint32_t FINISH_SPIN_LIMIT = 1u << 21;   // polls of about 2 us each

// STAGED: the block copies its rows of the rank-ordered bitmap into LDS first (PERMUTE_ROWS x Wr words) and serves a
// long run of tokens from there: 64 lanes that look 64 unrelated ranks up in global memory are 64 cache-line requests
// per instruction, which is what bounded the unstaged version (5 us at 16 rows, 16 us at 64).  The unstaged version
// remains for vocabularies whose rows do not fit LDS and for small batches.
template <bool STAGED>
__global__ __launch_bounds__(FINISH_BLOCK) void finish_kernel(MaskArgs a, uint32_t tokens_per_block, uint32_t row_groups) {
    extern __shared__ __align__(16) uint32_t rows_lds[];
    const DeviceTables &D = a.tab;
    const uint32_t tid = threadIdx.x, lane = tid & 63, Wr = (uint32_t)D.Wr;
    const uint32_t v_begin = blockIdx.x * tokens_per_block;            // a multiple of 64: a wavefront's ballot is two whole words
    const uint32_t v_end = v_begin + tokens_per_block < (uint32_t)D.V ? v_begin + tokens_per_block : (uint32_t)D.V;
    constexpr int AHEAD = STAGED ? PERMUTE_AHEAD : 1;
    uint32_t r_first[AHEAD];                              // requested alongside the fallback count: they do not depend on it
#pragma unroll
    for (int u = 0; u < AHEAD; u++) {
        const uint32_t v = v_begin + (uint32_t)u * FINISH_BLOCK + tid;
        r_first[u] = v < v_end ? D.rank_of[v] : 0xFFFFFFFFu;
    }
    const uint32_t n_blocks = gridDim.x * gridDim.y;
    const uint32_t n_over = a.counters[0];
    if (n_over != 0) {
        const uint32_t lin = blockIdx.y * gridDim.x + blockIdx.x;
        const uint32_t fb_waves = n_blocks * FINISH_WAVES < a.fb_waves ? n_blocks * FINISH_WAVES : a.fb_waves;
        const uint32_t gw = lin * FINISH_WAVES + (tid >> 6);
        if (gw < fb_waves) {
            fallback_wave(a, gw, fb_waves, n_over, lane);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // its verdict bits and error counts before its count
            if (lane == 0) atomicAdd(&a.counters[4], 1u);
        }
        if (tid == 0) {
            uint32_t spins = 0;
            while (__hip_atomic_load(&a.counters[4], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < fb_waves) {
                __builtin_amdgcn_s_sleep(64);
                if (++spins > FINISH_SPIN_LIMIT) { atomicAdd(&a.counters[2], 1u); __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); break; }
            }
        }
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    for (uint32_t rg = blockIdx.y; rg < row_groups; rg += gridDim.y) {
        const uint32_t row0 = rg * PERMUTE_ROWS;
        const uint32_t n_rows = (uint32_t)a.batch - row0 < (uint32_t)PERMUTE_ROWS ? (uint32_t)a.batch - row0 : (uint32_t)PERMUTE_ROWS;
        uint32_t r_ahead[AHEAD];
#pragma unroll
        for (int u = 0; u < AHEAD; u++) r_ahead[u] = r_first[u];
        const uint32_t *rows = a.rank_mask + (size_t)row0 * Wr;           // the group's rows are neighbours in memory
        if (STAGED) {
            if (rg != blockIdx.y) __syncthreads();                        // the previous group's readers are done with the LDS copy
            const uint32_t n_words = n_rows * Wr, n16 = n_words / 4;
            const uint4 *src = reinterpret_cast<const uint4 *>(rows);     // row0 * Wr * 4 bytes: 16-byte aligned when Wr is a multiple of 4
            if (((size_t)row0 * Wr) % 4 == 0) {
                for (uint32_t k = tid; k < n16; k += FINISH_BLOCK) reinterpret_cast<uint4 *>(rows_lds)[k] = src[k];
                for (uint32_t k = n16 * 4 + tid; k < n_words; k += FINISH_BLOCK) rows_lds[k] = rows[k];
            } else {
                for (uint32_t k = tid; k < n_words; k += FINISH_BLOCK) rows_lds[k] = rows[k];
            }
            __syncthreads();
            rows = rows_lds;
        }
        for (uint32_t v0 = v_begin; v0 < v_end; v0 += AHEAD * FINISH_BLOCK) {
            uint32_t r_next[AHEAD];
#pragma unroll
            for (int u = 0; u < AHEAD; u++) {                              // the next round's ranks are requested before this round's are used
                const uint32_t v = v0 + (uint32_t)(AHEAD + u) * FINISH_BLOCK + tid;
                r_next[u] = v < v_end ? D.rank_of[v] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u = 0; u < AHEAD; u++) {
                const uint32_t v = v0 + (uint32_t)u * FINISH_BLOCK + tid, r = r_ahead[u];
                if (v0 + (uint32_t)u * FINISH_BLOCK >= v_end) break;      // uniform over the block
                uint32_t word[PERMUTE_ROWS];
#pragma unroll
                for (int k = 0; k < PERMUTE_ROWS; k++)                     // all rows' words are requested before the first one is used
                    word[k] = (r != 0xFFFFFFFFu && (uint32_t)k < n_rows) ? rows[(size_t)k * Wr + (r >> 5)] : 0u;
                const uint32_t w = v >> 5;
#pragma unroll
                for (int k = 0; k < PERMUTE_ROWS; k++) {
                    const unsigned long long b = __ballot((word[k] >> (r & 31)) & 1u);
                    if ((uint32_t)k < n_rows && (lane & 31) == 0 && v < v_end)   // v is the word's first token; words past the block's run belong to the next block
                        a.out_mask[(size_t)(a.dst_row ? a.dst_row[row0 + k] : row0 + k) * D.W + w] = (uint32_t)(b >> lane);
                }
            }
#pragma unroll
            for (int u = 0; u < AHEAD; u++) r_ahead[u] = r_next[u];
        }
    }
    if (a.handoff_in_permute) hand_over(a, blockIdx.y * gridDim.x + blockIdx.x, n_blocks, n_over != 0);
}

}  // namespace

int choose_table_mode(const DeviceTables &t) {
    if (table_bytes(t, 0) <= (uint32_t)TABLE_LDS_BUDGET) return 0;
    if (table_bytes(t, 1) <= (uint32_t)TABLE_LDS_BUDGET) return 1;
    return 2;
}

hipError_t prepare_walk_kernels() {
    const int max_lds = 160 * 1024;
    hipError_t e;
#define SET_ATTR(k) if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k), hipFuncAttributeMaxDynamicSharedMemorySize, max_lds)) != hipSuccess) return e
    SET_ATTR(mask_walk_kernel<0>); SET_ATTR(mask_walk_kernel<1>); SET_ATTR(mask_walk_kernel<2>);
#undef SET_ATTR
    // the closing kernel also has a static word of LDS (hand_over): leave room for it below the 160 KB
    if ((e = hipFuncSetAttribute(reinterpret_cast<const void *>(&finish_kernel<true>), hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024)) != hipSuccess) return e;
    return hipSuccess;
}

hipError_t launch_cache_merge(const MaskArgs &a, hipStream_t s) {
    dim3 grid(((a.tab.Wr + 1) / 2 + 255) / 256, a.batch);
    hipLaunchKernelGGL(cache_merge_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}
uint32_t walk_lds_bytes(const DeviceTables &t, int mode, int lane_cap) {
    return table_bytes(t, mode) + 16 + WALK_WAVES * wave_region_bytes((uint32_t)lane_cap);
}
// Blocks of the walk kernel one compute unit holds at once (registers and LDS both limit it): the
// persistent grid must not be larger, or the surplus blocks would start only after others finish.
hipError_t walk_blocks_per_cu(int mode, uint32_t lds_bytes, int *out) {
    int n = 0;
    hipError_t e;
    if (mode == 0) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_walk_kernel<0>, WALK_BLOCK, lds_bytes);
    else if (mode == 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_walk_kernel<1>, WALK_BLOCK, lds_bytes);
    else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, mask_walk_kernel<2>, WALK_BLOCK, lds_bytes);
    *out = n < 1 ? 1 : n;
    return e;
}
hipError_t launch_mask_walk(const MaskArgs &a, hipStream_t s) {
    const uint32_t lds = walk_lds_bytes(a.tab, a.mode, a.lane_cap);
    dim3 grid(a.walk_blocks);
    if (a.mode == 0) hipLaunchKernelGGL(mask_walk_kernel<0>, grid, dim3(WALK_BLOCK), lds, s, a);
    else if (a.mode == 1) hipLaunchKernelGGL(mask_walk_kernel<1>, grid, dim3(WALK_BLOCK), lds, s, a);
    else hipLaunchKernelGGL(mask_walk_kernel<2>, grid, dim3(WALK_BLOCK), lds, s, a);
    return hipGetLastError();
}
hipError_t launch_finish(const MaskArgs &a, int cus, hipStream_t s) {
    const uint32_t row_groups = (uint32_t)(a.batch + PERMUTE_ROWS - 1) / PERMUTE_ROWS;
    const uint32_t lds = (uint32_t)PERMUTE_ROWS * (uint32_t)a.tab.Wr * 4u;
    const uint32_t n_cu = (uint32_t)(cus > 0 ? cus : 256);
    // staged: about four blocks per compute unit, each serving a run of tokens (a multiple of 64) from its LDS copy of the rows;
    // unstaged: one block per 256 tokens, one token per thread.  Staging pays when a block's run is long enough to earn the copy
    // back: from 1024 tokens on, with four blocks per compute unit (config 3, 16 rows: 5.1 us unstaged, 5.9 us staged with runs
    // of 512; config 4, 64 rows: 13.4 us unstaged, 9.4 us staged with runs of 2016; one, two, eight blocks per unit: 16.2, 11.4, 12.2 us).
    uint32_t x_blocks = ((uint32_t)a.tab.V + FINISH_BLOCK - 1) / FINISH_BLOCK;
    const uint32_t want = (4u * n_cu + row_groups - 1) / row_groups;
    const bool staged = lds <= 150u * 1024u && (uint32_t)a.tab.V / (want > 0 ? want : 1u) >= 1024u;
    if (staged && want < x_blocks) x_blocks = want;
    if (x_blocks < 1) x_blocks = 1;
    // The chip must hold the whole grid at once (blocks may wait for the fallback wavefronts of other blocks): ask the runtime how
    // many blocks a compute unit takes, and let blocks loop over row groups, then over longer token runs, when there are more.
    static int occ[2] = {0, 0};
    static uint32_t occ_lds = 0xFFFFFFFFu;
    if (!occ[staged] || (staged && occ_lds != lds)) {
        int n = 0;
        const hipError_t e = staged ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, finish_kernel<true>, FINISH_BLOCK, lds)
                                    : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, finish_kernel<false>, FINISH_BLOCK, 0);
        if (e != hipSuccess) return e;
        occ[staged] = n < 1 ? 1 : n;
        if (staged) occ_lds = lds;
    }
    const uint32_t cap = (uint32_t)occ[staged] * n_cu;
    uint32_t y_blocks = row_groups;
    if (x_blocks * y_blocks > cap) {
        y_blocks = cap / x_blocks < 1 ? 1 : (cap / x_blocks < row_groups ? cap / x_blocks : row_groups);
        if (x_blocks * y_blocks > cap) x_blocks = cap;           // a single row group per pass and still too many blocks: longer token runs
    }
    uint32_t tokens_per_block = (((uint32_t)a.tab.V + x_blocks - 1) / x_blocks + (staged ? 63u : (uint32_t)FINISH_BLOCK - 1)) & ~(staged ? 63u : (uint32_t)FINISH_BLOCK - 1);
    if (tokens_per_block < 64) tokens_per_block = 64;
    x_blocks = ((uint32_t)a.tab.V + tokens_per_block - 1) / tokens_per_block;
    if (x_blocks < 1) x_blocks = 1;
    dim3 grid(x_blocks, y_blocks);
    if (staged) hipLaunchKernelGGL(finish_kernel<true>, grid, dim3(FINISH_BLOCK), lds, s, a, tokens_per_block, row_groups);
    else hipLaunchKernelGGL(finish_kernel<false>, grid, dim3(FINISH_BLOCK), 0, s, a, tokens_per_block, row_groups);
    return hipGetLastError();
}
}  // namespace zf
