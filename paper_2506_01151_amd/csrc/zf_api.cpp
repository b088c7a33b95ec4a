// The C boundary: argument checks, engine / state life cycle, advance, chart packing and
// upload, kernel launches.
#include <hip/hip_runtime_api.h>
#include <unistd.h>
#include <algorithm>
#include <chrono>
#include <atomic>
#include <condition_variable>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <thread>
#include <unordered_map>
#include <unordered_set>
#include "zf_internal.h"
#include "zf_host_automaton.h"
#include "zf_launch.h"

using namespace zf;

namespace zf {
static thread_local std::string g_err;
void set_error(const std::string &m) { g_err = m; }
// Bring the state's chart up to date: the bytes fed through the host automaton since it last was, one zf_advance call at
// a time (Scan -> Complete -> Compact -> Predict, as feed_token_bytes does without the automaton).
static void catch_up(zf_state *s) {
    if (s->lag.empty()) return;
    const Tables &t = s->eng->tab;
    Chart &c = s->chart;
    int64_t created = 0;
    size_t at = 0;
    for (uint32_t cut : s->lag_cut) {
        for (; at < cut; at++) (void)earley_step(t, c, s->lag[at], false, &created);
        chart_compact(t, c);
    }
    s->items_created += created;
    s->lag.clear(); s->lag_cut.clear();
}
const Chart &chart_of(const zf_state *s) {
    catch_up(const_cast<zf_state *>(s));
    return s->chart;
}

}  // namespace zf

// Device-side resources of an engine.
struct DeviceSide {
    int device = 0;
    DeviceTables tab{};
    std::vector<void *> owned;           // table allocations
    // per-call buffers, grown on demand
    void *d_chart = nullptr; size_t chart_cap = 0;
    static const int N_SLOTS = 4;                    // calls that may be in flight before zf_mask_wait
    void *h_stage[N_SLOTS] = {nullptr, nullptr, nullptr, nullptr}; size_t stage_cap[N_SLOTS] = {0, 0, 0, 0};   // pinned
    hipEvent_t stage_done[N_SLOTS] = {nullptr, nullptr, nullptr, nullptr};   // the slot's upload has been consumed
    uint32_t *h_status = nullptr;                    // pinned, [N_SLOTS][8]: counters [0..3] and the call's number [4], written by each call's last kernel
    uint32_t call_seq = 0, last_seq = 0, last_slot = 0; // number of the newest call in flight and its slot
    uint32_t next_slot = 0, pending = 0;
    uint32_t occ_lds = 0;                            // LDS size the cached occupancy answer belongs to
    int occ_blocks = 1;
    // State cache (paper Section 5.2): finished token-order mask rows keyed by the row's packed chart.
    struct CacheEntry { uint64_t hash = 0; std::vector<uint32_t> key; uint32_t stamp = 0; bool used = false; };
    std::vector<CacheEntry> cache;                   // one per pool slot
    std::unordered_multimap<uint64_t, uint32_t> cache_index;
    uint32_t *d_pool = nullptr;                      // [cache.size()][W]
    uint32_t cache_victim = 0, cache_call = 0;
    uint32_t *d_rank_mask = nullptr; size_t rank_cap = 0;
    uint4 *d_overflow = nullptr; size_t overflow_cap = 0;
    uint4 *d_work = nullptr;
    int cus = 256;
    int mode = 2;
    uint32_t *d_counters = nullptr;
    uint2 *d_fb_items = nullptr;
    uint32_t *d_fb_ss = nullptr;
    uint8_t *scratch = nullptr;          // this device's copy of the static array behind zf_compute_mask_noalloc
    // The persistent automaton (walk_mode 2).
    StoreView store{};
    void *d_root_items = nullptr; uint32_t n_root = 0;
    uint32_t *d_import_root = nullptr;               // [MAX_BATCH]
    uint32_t *h_row_out = nullptr;                   // pinned, [N_SLOTS][MAX_BATCH]: the state each row of a call ends up in
    uint32_t *d_row_out = nullptr;                   // the same in device memory: the mask kernel writes here, the call's last block copies it out
    uint32_t store_epoch = 1;                        // bumped whenever the store is cleared
    uint32_t store_states = 0, store_items = 0;      // as of the last call that reported back
    bool store_dirty = true;                         // the store must be cleared before its next use
    // What sizes a call's grid: the tokens a row's token-mask cache rows leave to the parser.  The host keeps the token-order
    // rows and counts the union for every set of cache rows it meets, once (a few microseconds; the sets repeat all the time).
    std::vector<uint32_t> h_valid_tok, h_cd_tok;     // [Q + N][W]
    std::unordered_map<uint64_t, uint32_t> undecided_of;   // signature of the list of cache rows -> undecided tokens
    uint32_t store_backoff = 0, store_backoff_next = 8;   // after a call the store had no room for: calls that take the per-block automaton instead
    struct CallRecord {                              // what to note in the states once the call in this slot has reported
        bool active = false;
        uint32_t epoch = 0;
        std::vector<std::shared_ptr<StateLink>> st; std::vector<uint32_t> gen; std::vector<uint64_t> upto;
        std::vector<uint64_t> hop;                   // per row: the (state, token) pair the kernel walks, to be noted with the state it reports; 0 = none
        std::vector<uint32_t> host;                  // per row: the state's name in the host automaton, to be noted with the name the kernel reports; 0 = none
        uint32_t host_epoch = 0;                     // ... and the epoch of the host automaton that name belongs to
    } rec[N_SLOTS];
    // The device's name of a state of the host automaton, as the mask kernel has reported it for a row that stood there.  The two
    // automata hold the same sets under different names; once a state's device name is known, a row that arrives in it is sent
    // with that name and no bytes to walk, whatever token took it there.  Valid while neither automaton has been emptied.
    std::vector<uint32_t> name_of_host;
    uint32_t name_host_epoch = 0, name_store_epoch = 0;
    uint32_t name_find(uint32_t host_id, uint32_t host_epoch, uint32_t st_epoch) const {   // 0 = unknown
        return host_epoch == name_host_epoch && st_epoch == name_store_epoch && host_id < name_of_host.size() ? name_of_host[host_id] : 0u;
    }
    void name_note(uint32_t host_id, uint32_t host_epoch, uint32_t st_epoch, uint32_t dev) {
        if (host_epoch != name_host_epoch || st_epoch != name_store_epoch) { name_of_host.clear(); name_host_epoch = host_epoch; name_store_epoch = st_epoch; }
        if (host_id >= (1u << 22)) return;
        if (host_id >= name_of_host.size()) name_of_host.resize(std::max<size_t>(host_id + 1, name_of_host.size() * 2), 0u);
        name_of_host[host_id] = dev;
    }
    // Where a token leads from a state of the persistent automaton, as the mask kernel has reported it: (state << 32 | token + 1)
    // -> state.  Names are stable while the store is not cleared, so a row that is fed a token in a state some row was fed it in
    // before is sent with the state it arrives in and no bytes to walk.  Open addressing, exact keys, emptied with the store.
    std::vector<uint64_t> hop_key; std::vector<uint32_t> hop_val;
    uint32_t hop_used = 0, hop_epoch = 0;
    static const uint32_t HOP_SLOTS = 1u << 16;
    uint32_t hop_find(uint64_t key) const {          // 0 = unknown
        if (hop_key.empty()) return 0;
        for (uint32_t i = (uint32_t)((key * 0x9E3779B97F4A7C15ull) >> 48);; i = (i + 1) & (HOP_SLOTS - 1)) {
            if (hop_key[i] == key) return hop_val[i];
            if (hop_key[i] == 0) return 0;
        }
    }
    void hop_note(uint64_t key, uint32_t val) {
        if (hop_key.empty()) { hop_key.assign(HOP_SLOTS, 0); hop_val.assign(HOP_SLOTS, 0); }
        if (hop_used >= HOP_SLOTS / 2) { std::fill(hop_key.begin(), hop_key.end(), 0); hop_used = 0; }
        for (uint32_t i = (uint32_t)((key * 0x9E3779B97F4A7C15ull) >> 48);; i = (i + 1) & (HOP_SLOTS - 1)) {
            if (hop_key[i] == key) return;
            if (hop_key[i] == 0) { hop_key[i] = key; hop_val[i] = val; hop_used++; return; }
        }
    }
    zf_mask_report report{};
    uint32_t call_parity = 0;            // which of the two counter sets the next call uses
    bool profiling = false;
    bool closing_kernel = true;          // the last call enqueued a kernel behind its mask kernel (closing kernel or gather)
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
};

namespace {

const int MAX_BATCH = 4096;   // rows per zf_compute_mask call
const uint32_t STORE_ROOT_ID = 1;

int fail(int code, const std::string &m) { set_error(m); return code; }
#define HIP_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return fail(ZF_ERR_DEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); } while (0)

template <class Tv>
int upload(DeviceSide *d, const std::vector<Tv> &v, const Tv **out, uint32_t *bytes_out = nullptr) {
    // padded to a multiple of 16 bytes (zero filled) so that blocks can stage it with 16-byte copies
    void *p = nullptr;
    size_t bytes = (std::max<size_t>(v.size() * sizeof(Tv), 16) + 15) & ~(size_t)15;
    HIP_TRY(hipMalloc(&p, bytes));
    d->owned.push_back(p);
    HIP_TRY(hipMemset(p, 0, bytes));
    if (!v.empty()) HIP_TRY(hipMemcpy(p, v.data(), v.size() * sizeof(Tv), hipMemcpyHostToDevice));
    *out = (const Tv *)p;
    if (bytes_out) *bytes_out = (uint32_t)bytes;
    return ZF_OK;
}

void free_device(DeviceSide *d) {
    if (!d) return;
    (void)hipSetDevice(d->device);
    for (void *p : d->owned) (void)hipFree(p);
    if (d->d_chart) (void)hipFree(d->d_chart);
    for (int k = 0; k < DeviceSide::N_SLOTS; k++) { if (d->h_stage[k]) (void)hipHostFree(d->h_stage[k]); if (d->stage_done[k]) (void)hipEventDestroy(d->stage_done[k]); }
    if (d->h_status) (void)hipHostFree(d->h_status);
    if (d->d_pool) (void)hipFree(d->d_pool);
    if (d->d_rank_mask) (void)hipFree(d->d_rank_mask);
    if (d->d_overflow) (void)hipFree(d->d_overflow);
    if (d->d_work) (void)hipFree(d->d_work);
    if (d->d_counters) (void)hipFree(d->d_counters);
    if (d->d_fb_items) (void)hipFree(d->d_fb_items);
    if (d->d_fb_ss) (void)hipFree(d->d_fb_ss);
    if (d->store.hdr) (void)hipFree(d->store.hdr);
    if (d->store.arena) (void)hipFree(d->store.arena);
    if (d->store.trans) (void)hipFree(d->store.trans);
    if (d->store.intern) (void)hipFree(d->store.intern);
    if (d->store.ctl) (void)hipFree(d->store.ctl);
    if (d->d_root_items) (void)hipFree(d->d_root_items);
    if (d->d_import_root) (void)hipFree(d->d_import_root);
    if (d->h_row_out) (void)hipHostFree(d->h_row_out);
    if (d->d_row_out) (void)hipFree(d->d_row_out);
    for (auto &ev : d->ev) if (ev) (void)hipEventDestroy(ev);
    delete d;
}

int setup_device(zf_engine *e) {
    DeviceSide *d = new (std::nothrow) DeviceSide();
    if (!d) return fail(ZF_ERR_OOM, "out of memory");
    e->dev = d;
    d->device = e->opt.device;
    HIP_TRY(hipSetDevice(d->device));
    const Tables &t = e->tab;
    const Trie &tr = e->trie;
    DeviceTables &T = d->tab;
    int rc;
    std::vector<uint8_t> cls(t.cls, t.cls + 256);
#define UP(field, vec, bytes) if ((rc = upload(d, vec, &T.field, bytes)) != ZF_OK) return rc
    {   // the grammar tables in one allocation, in the order the kernels lay them out in LDS, each padded
        // to 16 bytes: a block stages whatever prefix fits with one flat copy
        std::vector<uint8_t> blob;
        size_t at[8];
        auto add = [&](const void *p, size_t bytes, uint32_t *padded, int k) {
            at[k] = blob.size();
            const size_t pad = (std::max<size_t>(bytes, 16) + 15) & ~(size_t)15;
            blob.resize(blob.size() + pad, 0);
            if (bytes) memcpy(blob.data() + at[k], p, bytes);
            *padded = (uint32_t)pad;
        };
        add(t.advpq.data(), t.advpq.size() * 4, &T.small_bytes[0], 0); add(cls.data(), cls.size(), &T.small_bytes[1], 1);
        add(t.qinfo.data(), t.qinfo.size() * 4, &T.small_bytes[2], 2); add(t.scan_off.data(), t.scan_off.size() * 4, &T.small_bytes[3], 3);
        add(t.comp_off.data(), t.comp_off.size() * 4, &T.small_bytes[4], 4);
        add(t.delta_dense.data(), t.delta_dense.size() * 4, &T.big_bytes[0], 5); add(t.dev_scan_list.data(), t.dev_scan_list.size() * 4, &T.big_bytes[1], 6);
        add(t.dev_comp_list.data(), t.dev_comp_list.size() * 4, &T.big_bytes[2], 7);
        const uint8_t *dev = nullptr;
        if ((rc = upload(d, blob, &dev)) != ZF_OK) return rc;
        T.table_blob = dev;
        T.advpq = (const uint32_t *)(dev + at[0]); T.cls = dev + at[1]; T.qinfo = (const uint32_t *)(dev + at[2]);
        T.scan_off = (const uint32_t *)(dev + at[3]); T.comp_off = (const uint32_t *)(dev + at[4]); T.delta = (const uint32_t *)(dev + at[5]);
        T.scan_list = (const uint32_t *)(dev + at[6]); T.comp_list = (const uint32_t *)(dev + at[7]);
    }
    UP(nodes, tr.nodes, nullptr); UP(parent, tr.parent, nullptr); UP(chunk_begin, tr.chunk_begin, nullptr); UP(chunk_end, tr.chunk_end, nullptr);
    UP(chunk_anc, tr.chunk_anc, nullptr); UP(rank_of, tr.rank_of, nullptr);
    UP(ci_valid, tr.ci_valid, nullptr); UP(ci_cd, tr.ci_cd, nullptr);
    {   // the strings as class strings for the mask-automaton kernel
        std::vector<uint8_t> str_cls(tr.str_bytes.size()), rep(std::max(t.n_cls, 1), 0);
        for (size_t k = 0; k < tr.str_bytes.size(); k++) str_cls[k] = t.cls[tr.str_bytes[k]];
        for (int b = 255; b >= 0; b--) rep[t.cls[b]] = (uint8_t)b;
        std::vector<Str16> str16((size_t)std::max(tr.n_strings, 1), Str16{{0, 0, 0, 0}});
        for (int r = 0; r < tr.n_strings; r++) {
            uint8_t first[16] = {0};
            const uint32_t n = std::min<uint32_t>(16, tr.str_off[r + 1] - tr.str_off[r]);
            memcpy(first, str_cls.data() + tr.str_off[r], n);
            memcpy(&str16[r], first, 16);
        }
        UP(str_off, tr.str_off, nullptr); UP(str_cls, str_cls, nullptr); UP(str16, str16, nullptr); UP(cls_rep, rep, nullptr);
    }
    if (e->store_on) {
        // The mask kernel over the persistent automaton works in token order: every token's string as byte classes, and the
        // rows of the token-mask cache with one bit per token (bit v = the rank-ordered row's bit for token v's string).
        const size_t V = (size_t)e->V, W = (size_t)e->W, n_rows = tr.Wr > 0 ? tr.ci_valid.size() / (size_t)tr.Wr : 0;
        std::vector<Str16> tok16(std::max<size_t>(V, 1), Str16{{0, 0, 0, 0}});
        std::vector<uint8_t> tok_len(std::max<size_t>(V, 1), 0);
        for (size_t v = 0; v < V; v++) {
            const uint32_t r = tr.rank_of[v];
            if (r == 0xFFFFFFFFu) continue;
            const uint32_t n = tr.str_off[r + 1] - tr.str_off[r];
            uint8_t first[16] = {0};
            for (uint32_t k = 0; k < std::min<uint32_t>(16, n); k++) first[k] = t.cls[tr.str_bytes[tr.str_off[r] + k]];
            memcpy(&tok16[v], first, 16);
            tok_len[v] = n <= 16 ? (uint8_t)n : (uint8_t)TOK_LEN_LONG;
        }
        std::vector<uint32_t> &valid_tok = d->h_valid_tok, &cd_tok = d->h_cd_tok;
        valid_tok.assign(std::max<size_t>(n_rows * W, 1), 0); cd_tok.assign(std::max<size_t>(n_rows * W, 1), 0);
        auto rows_job = [&](size_t r0, size_t r1) {
            for (size_t r = r0; r < r1; r++) {
                const uint32_t *sv = &tr.ci_valid[r * tr.Wr], *sc = &tr.ci_cd[r * tr.Wr];
                uint32_t *dv = &valid_tok[r * W], *dc = &cd_tok[r * W];
                for (size_t v = 0; v < V; v++) {
                    const uint32_t k = tr.rank_of[v];
                    if (k == 0xFFFFFFFFu) continue;
                    const uint32_t bv = (sv[k >> 5] >> (k & 31)) & 1u, bc = (sc[k >> 5] >> (k & 31)) & 1u;
                    dv[v >> 5] |= bv << (v & 31);
                    dc[v >> 5] |= bc << (v & 31);
                }
            }
        };
        const size_t n_thr = std::min<size_t>(std::max<size_t>(1, std::min<unsigned>(8, std::thread::hardware_concurrency())), std::max<size_t>(n_rows, 1));
        if (n_thr <= 1 || n_rows * V < (size_t)1 << 22) rows_job(0, n_rows);
        else {
            std::vector<std::thread> pool;
            for (size_t k = 0; k < n_thr; k++) pool.emplace_back(rows_job, n_rows * k / n_thr, n_rows * (k + 1) / n_thr);
            for (auto &th : pool) th.join();
        }
        UP(tok16, tok16, nullptr); UP(tok_len, tok_len, nullptr); UP(ci_valid_tok, valid_tok, nullptr); UP(ci_cd_tok, cd_tok, nullptr);
    }
    T.Q = t.Q;
#undef UP
    T.N = t.N; T.n_cls = t.n_cls; T.end_base = t.end_base; T.n_nodes = (int)tr.nodes.size(); T.n_chunks = (int)tr.chunk_begin.size();
    T.n_strings = tr.n_strings; T.V = e->V; T.W = e->W; T.chunk_ranks = tr.chunk_ranks;
    T.Wr = tr.Wr;
    d->mode = choose_table_mode(T);
    HIP_TRY(prepare_kernels());
    HIP_TRY(hipDeviceGetAttribute(&d->cus, hipDeviceAttributeMultiprocessorCount, d->device));
    if (e->opt.state_cache_entries > 0 && e->W > 0) {
        d->cache.resize(e->opt.state_cache_entries);
        HIP_TRY(hipMalloc((void **)&d->d_pool, (size_t)e->opt.state_cache_entries * e->W * 4));
    }
    if (walk_lds_bytes(T, d->mode, e->opt.lane_item_cap) > 160u * 1024u)
        return fail(ZF_ERR_INVALID_ARG, "lane_item_cap and the grammar tables do not fit the 160 KB of LDS");
    HIP_TRY(hipMalloc((void **)&d->d_counters, 2 * COUNTER_SET_WORDS * 4));     // two sets of counters (see MaskArgs::counters)
    HIP_TRY(hipMemset(d->d_counters, 0, 2 * COUNTER_SET_WORDS * 4));
    HIP_TRY(hipHostMalloc((void **)&d->h_status, 32 * DeviceSide::N_SLOTS, hipHostMallocDefault));
    memset(d->h_status, 0, 32 * DeviceSide::N_SLOTS);
    for (auto &ev : d->stage_done) HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    for (int k = 0; k < DeviceSide::N_SLOTS; k++) {     // staging room every engine has from the start (zf_compute_mask_noalloc never grows it)
        HIP_TRY(hipHostMalloc(&d->h_stage[k], NOALLOC_STAGE_BYTES, hipHostMallocDefault));
        d->stage_cap[k] = NOALLOC_STAGE_BYTES;
    }
    if (e->store_on) {
        // Room of the persistent automaton: states x byte classes transition words (at most 128 MB), 4 M items, a hash table of
        // twice as many slots as states.  The host clears the store when it is half full (see enqueue_mask_impl).
        StoreView &G = d->store;
        uint32_t cap = 1u << 18;
        while (cap > 4096 && (size_t)cap * (size_t)std::max(t.n_cls, 1) * 4 > ((size_t)128 << 20)) cap >>= 1;
        G.cap_states = cap; G.cap_items = 1u << 22; G.intern_mask = 2 * cap - 1;
        HIP_TRY(hipMalloc((void **)&G.hdr, (size_t)G.cap_states * sizeof(uint2)));
        HIP_TRY(hipMalloc((void **)&G.arena, (size_t)G.cap_items * sizeof(uint2)));
        HIP_TRY(hipMalloc((void **)&G.trans, (size_t)G.cap_states * std::max(t.n_cls, 1) * 4));
        HIP_TRY(hipMalloc((void **)&G.intern, ((size_t)G.intern_mask + 1) * 8));
        HIP_TRY(hipMalloc((void **)&G.ctl, 64));
        HIP_TRY(hipMalloc((void **)&d->d_import_root, (size_t)MAX_BATCH * 4));
        HIP_TRY(hipHostMalloc((void **)&d->h_row_out, (size_t)DeviceSide::N_SLOTS * MAX_BATCH * 4, hipHostMallocDefault));
        HIP_TRY(hipMalloc((void **)&d->d_row_out, (size_t)DeviceSide::N_SLOTS * MAX_BATCH * 4));
        HIP_TRY(hipMemset(d->d_row_out, 0, (size_t)DeviceSide::N_SLOTS * MAX_BATCH * 4));
        Chart c0;                                        // the empty prefix's set, completed items dropped, as device item words
        chart_init(t, c0);
        std::vector<uint32_t> root;
        for (const Item &it : c0.items) {
            if ((t.sym[it.p] >> SYM_KIND_SHIFT) == SYM_END) continue;
            const uint32_t aw = t.advpq[it.p];
            root.push_back((aw & IW_TERM) ? ((aw & 0xFFFFu) | ((uint32_t)it.q << 16)) : aw);
            root.push_back(0);
        }
        d->n_root = (uint32_t)root.size() / 2;
        HIP_TRY(hipMalloc(&d->d_root_items, std::max<size_t>(root.size() * 4, 16)));
        if (!root.empty()) HIP_TRY(hipMemcpy(d->d_root_items, root.data(), root.size() * 4, hipMemcpyHostToDevice));
        d->store_dirty = true;
    }
    HIP_TRY(scratch_init(d->device));                    // once per device, with that device current
    d->scratch = (uint8_t *)scratch_ptr(d->device);
    if (!d->scratch) return fail(ZF_ERR_DEVICE, "the device address of the static scratch array is unknown");
    HIP_TRY(hipMalloc((void **)&d->d_fb_items, (size_t)FB_ITEMS_PER_WAVE * FB_WAVES * sizeof(uint2)));
    HIP_TRY(hipMalloc((void **)&d->d_fb_ss, (size_t)(FB_DEPTH_MAX + 2) * FB_WAVES * sizeof(uint32_t)));
    return ZF_OK;
}

// Rows of the token-mask cache that the items of the current set select: the DFA state of an
// item that stands inside (or before) a terminal, Q + Y for an item that waits for nonterminal Y.
uint32_t current_set_entries(const Tables &t, const Item *items, uint32_t n_items, uint32_t *out) {
    uint32_t n = 0;
    for (uint32_t i = 0; i < n_items; i++) {
        uint16_t code = t.sym[items[i].p];
        uint32_t row;
        if ((code >> SYM_KIND_SHIFT) == SYM_TERM) row = items[i].q;
        else if ((code >> SYM_KIND_SHIFT) == SYM_NT) row = (uint32_t)t.Q + (code & SYM_ID_MASK_NT);
        else continue;
        bool dup = false;
        for (uint32_t k = 0; k < n && !dup; k++) dup = out[k] == row;
        if (!dup) out[n++] = row;
    }
    return n;
}
uint32_t current_set_entries(const Tables &t, const Chart &c, uint32_t *out) {
    const uint32_t lo = c.set_off[c.n_sets() - 1];
    return current_set_entries(t, c.items.data() + lo, c.set_off[c.n_sets()] - lo, out);
}

static const size_t HOST_LAG_MAX = 1u << 16;          // bytes a chart may lag behind before it is brought up to date anyway
static const int64_t HOST_AUT_ITEMS_MAX = 1 << 25;    // the host automaton is emptied when it is full or holds more items than this

// The state's place in the host automaton (the caller holds the engine's lock).
uint32_t host_place(zf_state *s) {
    zf_engine *e = s->eng;
    if (s->host_id == HostAutomaton::ROOT || s->host_id_epoch == e->host_epoch) return s->host_id;
    const uint32_t at = e->host_aut->import(chart_of(s));   // the automaton was emptied since: the chart says where the state stands
    if (at == 0) return 0;                             // no room
    s->host_id = at; s->host_id_epoch = e->host_epoch;
    return s->host_id;
}

// The items of the state's current set and the size of the largest set its chart holds -- from the host automaton when the
// engine has one (the caller holds its lock; the chart may lag behind), else from the chart.
struct CurrentSet { const Item *items; uint32_t n, biggest; };
CurrentSet current_set(zf_state *s) {
    zf_engine *e = s->eng;
    if (e->host_aut) {
        const uint32_t at = host_place(s);
        if (at == HostAutomaton::SINK) return CurrentSet{nullptr, 0, 0};
        if (at == 0) {                                     // the automaton has no room for the state's chart: the chart itself, then
            const Chart &c = chart_of(s);
            uint32_t biggest = 0;
            for (uint32_t k = 0; k < c.n_sets(); k++) biggest = std::max(biggest, c.set_off[k + 1] - c.set_off[k]);
            const uint32_t lo = c.set_off[c.n_sets() - 1];
            return CurrentSet{c.items.data() + lo, c.set_off[c.n_sets()] - lo, biggest};
        }
        const HostAutomaton &A = *e->host_aut;
        const HostAutomaton::State &hs = A.st(at);
        return CurrentSet{hs.items.data(), (uint32_t)hs.items.size(), hs.widest};
    }
    const Chart &c = s->chart;
    uint32_t biggest = 0;
    for (uint32_t k = 0; k < c.n_sets(); k++) biggest = std::max(biggest, c.set_off[k + 1] - c.set_off[k]);
    const uint32_t lo = c.set_off[c.n_sets() - 1];
    return CurrentSet{c.items.data() + lo, c.set_off[c.n_sets()] - lo, biggest};
}

int feed_token_bytes(zf_state *s, const uint8_t *bytes, int64_t n) {
    if (n <= 0) return fail(ZF_ERR_REJECTED, "an empty token is never allowed");
    const Tables &t = s->eng->tab;
    const bool pruning = s->eng->opt.pruning != 0;
    if (s->eng->host_aut) {
        // Through the host automaton: a look-up per byte once the transition is known (Sections 4.4, 5.2: nothing is parsed
        // twice), an Earley byte step the first time -- run on a private copy of the sets it reads, without the lock, so
        // that the rows of a batch can be fed by several threads.  All or nothing, as below.
        zf_engine *e = s->eng;
        HostAutomaton &A = *e->host_aut;
        std::unique_lock<std::mutex> lk(e->host_mu);
        while (A.full() || A.n_items > HOST_AUT_ITEMS_MAX) {   // start over; the states find their way back through their charts
            if (e->host_walkers == 0) { A.clear(); e->host_epoch++; break; }
            lk.unlock();                                  // somebody is at work on a transition (and waits for nobody): let them finish
            std::this_thread::yield();
            lk.lock();
        }
        if (s->host_id != HostAutomaton::ROOT && s->host_id_epoch != e->host_epoch) {
            lk.unlock();
            const Chart &c = chart_of(s);                 // the automaton was emptied since: the chart says where the state stands
            lk.lock();
            const uint32_t at = A.import(c);
            if (at == 0) return fail(ZF_ERR_OOM, "the chart is too large for the host automaton");
            s->host_id = at; s->host_id_epoch = e->host_epoch;
        }
        const uint32_t epoch = e->host_epoch;             // cannot change while this thread is a walker or holds the lock
        uint32_t at = s->host_id;
        bool accepted = false;
        for (int64_t i = 0; i < n; i++) {
            if (at == HostAutomaton::SINK) at = HostAutomaton::DEAD;
            else {
                const int cl = t.cls[bytes[i]];
                if (A.st(at).trans[cl] == HostAutomaton::NONE) {
                    static thread_local HostAutomaton::Work w;
                    e->host_walkers++;
                    lk.unlock();
                    A.lay_out(at, w);
                    const StepResult r = earley_step(t, w.c, bytes[i], false, nullptr);
                    lk.lock();
                    e->host_walkers--;
                    if (A.st(at).trans[cl] == HostAutomaton::NONE) A.record(at, cl, r, w);   // else somebody else has made it meanwhile
                }
                accepted = A.st(at).acc[cl] != 0;
                at = A.st(at).trans[cl];
            }
            if (at == HostAutomaton::DEAD || (at == HostAutomaton::SINK && i + 1 < n))
                return fail(ZF_ERR_REJECTED, "byte " + std::to_string(i) + " of the input cannot extend the prefix");
        }
        s->host_id = at; s->host_id_epoch = epoch;
        s->accepting = accepted;
        lk.unlock();
        s->bytes_fed += n;
        s->lag.insert(s->lag.end(), bytes, bytes + n);
        s->lag_cut.push_back((uint32_t)s->lag.size());
        if (s->lag.size() > HOST_LAG_MAX) catch_up(s);
    } else {
        Chart &c = s->chart;
        const uint32_t keep = c.n_sets();
        int64_t created = 0;
        bool accepted = false;
        for (int64_t i = 0; i < n; i++) {
            StepResult r = earley_step(t, c, bytes[i], !pruning, &created);
            accepted = r.accepted;
            // a byte is rejected when its set is empty; a completed sentence that cannot be extended
            // is still fine as the last byte
            if (!r.alive || (!r.kernel_nonempty && i + 1 < n)) {
                c.truncate(keep);
                return fail(ZF_ERR_REJECTED, "byte " + std::to_string(i) + " of the input cannot extend the prefix");
            }
        }
        s->accepting = accepted;
        s->items_created += created;
        s->bytes_fed += n;
        if (pruning) chart_compact(t, c);   // Compact: after Complete, before the next Predict
    }
    if (s->eng->store_on) {                               // the device walks the same bytes at the next mask call
        for (int64_t i = 0; i < n; i++) s->pending.push_back(t.cls[bytes[i]]);
        s->fed_total += (uint64_t)n;
        s->pending_token = -1;                            // zf_advance knows better
        if (s->pending.size() > (size_t)STORE_PENDING_MAX) {   // too far behind: the row comes in through its chart again
            s->pending.clear(); s->pending_base = s->fed_total; s->dev_id = 0; s->dev_epoch = 0;
        }
    }
    return ZF_OK;
}

}  // namespace

extern "C" {

const char *zf_strerror(int code) {
    switch (code) {
    case ZF_OK: return "ok";
    case ZF_ERR_INVALID_ARG: return "invalid argument";
    case ZF_ERR_GRAMMAR: return "invalid grammar";
    case ZF_ERR_REJECTED: return "input rejected by the grammar";
    case ZF_ERR_RANGE: return "token id out of range";
    case ZF_ERR_DEVICE: return "device error";
    case ZF_ERR_OOM: return "out of memory";
    case ZF_ERR_OVERFLOW: return "Earley set exceeded the fallback arena";
    }
    return "unknown error";
}
const char *zf_last_error(void) { return g_err.c_str(); }

static void explore_from_the_empty_prefix(zf_engine *e);

int zf_compile(const zf_grammar_desc *g, const zf_vocab_desc *v, const zf_options *opt, zf_engine **out) {
    if (!g || !v || !out || v->V < 0 || (v->V && !v->off)) return fail(ZF_ERR_INVALID_ARG, "null argument");
    for (int i = 0; i < v->V; i++) {
        int64_t n = v->off[i + 1] - v->off[i];
        if (n < 0 || n > MAX_TOKEN_LEN_ON_DEVICE) return fail(ZF_ERR_INVALID_ARG, "token " + std::to_string(i) + ": length must be 0..255");
    }
    zf_engine *e = new (std::nothrow) zf_engine();
    if (!e) return fail(ZF_ERR_OOM, "out of memory");
    e->opt = opt ? *opt : zf_options{1, 0, 0, 0, 0, 0, 0, 0, 0};
    e->lane_cap_auto = e->opt.lane_item_cap <= 0;
    if (e->opt.lane_item_cap <= 0) e->opt.lane_item_cap = LANE_CAP_DEFAULT;
    if (e->opt.lane_item_cap > LANE_CAP_MAX) e->opt.lane_item_cap = LANE_CAP_MAX;
    if (e->opt.fallback_item_cap <= 0 || e->opt.fallback_item_cap > FB_ITEMS_PER_WAVE) e->opt.fallback_item_cap = FB_ITEMS_PER_WAVE;
    if (e->opt.state_cache_entries == 0) e->opt.state_cache_entries = 2048;
    if (e->opt.state_cache_entries < 0) e->opt.state_cache_entries = 0;
    if (e->opt.state_cache_entries > 65536) e->opt.state_cache_entries = 65536;
    if (e->opt.chunk_strings != 8 && e->opt.chunk_strings != 16 && e->opt.chunk_strings != 32) e->opt.chunk_strings = 8;
    if (e->opt.precompute_states == 0) e->opt.precompute_states = 65536;
    if (e->opt.precompute_states < 0) e->opt.precompute_states = 0;
    try {
        if (!build_tables(g, e->tab)) { delete e; return ZF_ERR_GRAMMAR; }
        e->V = v->V; e->W = (v->V + 31) / 32;
        e->voc_off.assign(v->off, v->off + v->V + 1);
        e->voc_bytes.assign(v->bytes, v->bytes + v->off[v->V]);
        build_trie(v, e->opt.chunk_strings, e->tab.cls, e->trie);
        build_token_mask_cache(e->tab, e->trie);
    } catch (const std::bad_alloc &) { delete e; return fail(ZF_ERR_OOM, "out of memory"); }
    e->store_on = e->opt.device >= 0 && e->opt.walk_mode == 2 && e->opt.pruning != 0;
    if (e->opt.walk_mode == 2 && e->opt.pruning != 0) {
        e->host_aut = new (std::nothrow) HostAutomaton(e->tab);
        if (!e->host_aut) { delete e; return fail(ZF_ERR_OOM, "out of memory"); }
    }
    if (e->opt.device >= 0) {
        int rc = setup_device(e);
        if (rc != ZF_OK) { free_device(e->dev); delete e->host_aut; delete e; return rc; }
    }
    explore_from_the_empty_prefix(e);
    *out = e;
    return ZF_OK;
}

void zf_engine_destroy(zf_engine *e) {
    if (!e) return;
    free_device(e->dev);
    delete e->host_aut;
    delete e;
}

int zf_engine_get_info(const zf_engine *e, zf_engine_info *o) {
    if (!e || !o) return fail(ZF_ERR_INVALID_ARG, "null argument");
    o->V = e->V; o->W = e->W; o->n_nonterminals = e->tab.N; o->n_rules = e->tab.n_rules_kept; o->n_positions = e->tab.P;
    o->n_dfa_states = e->tab.Q; o->n_byte_classes = e->tab.n_cls; o->n_trie_nodes = (int)e->trie.nodes.size();
    o->n_strings = e->trie.n_strings; o->lane_item_cap = e->opt.lane_item_cap; o->device = e->opt.device;
    o->table_lds_mode = e->dev ? e->dev->mode : -1;
    return ZF_OK;
}

int zf_state_new(zf_engine *e, zf_state **out) {
    if (!e || !out) return fail(ZF_ERR_INVALID_ARG, "null argument");
    zf_state *s = new (std::nothrow) zf_state();
    if (!s) return fail(ZF_ERR_OOM, "out of memory");
    s->eng = e;
    s->link = std::make_shared<StateLink>(StateLink{s});
    *out = s;
    return zf_state_reset(s);
}

int zf_state_reset(zf_state *s) {
    if (!s) return fail(ZF_ERR_INVALID_ARG, "null argument");
    const Tables &t = s->eng->tab;
    chart_init(t, s->chart);
    // the empty prefix is a sentence iff the start symbol is nullable: then the initial set holds
    // the completed start rule; drop completed items as every later set does (pruning on)
    s->accepting = false;
    Chart &c = s->chart;
    size_t w = 0;
    for (size_t i = 0; i < c.items.size(); i++) {
        bool done = (t.sym[c.items[i].p] >> SYM_KIND_SHIFT) == SYM_END;
        if (done) s->accepting = true;
        if (!done || !s->eng->opt.pruning) c.items[w++] = c.items[i];
    }
    c.items.resize(w);
    c.set_off[1] = (uint32_t)w;
    s->items_created = 0; s->bytes_fed = 0;
    s->dev_id = STORE_ROOT_ID; s->dev_epoch = 0; s->generation++;
    s->pending.clear(); s->pending_base = s->fed_total; s->pending_token = -1;
    s->lag.clear(); s->lag_cut.clear();
    s->host_id = HostAutomaton::ROOT; s->host_id_epoch = 0;
    return ZF_OK;
}

int zf_state_clone(const zf_state *s, zf_state **out) {
    if (!s || !out) return fail(ZF_ERR_INVALID_ARG, "null argument");
    zf_state *c = new (std::nothrow) zf_state(*s);
    if (!c) return fail(ZF_ERR_OOM, "out of memory");
    c->link = std::make_shared<StateLink>(StateLink{c});
    *out = c;
    return ZF_OK;
}

void zf_state_destroy(zf_state *s) {
    if (s && s->link) s->link->s = nullptr;               // calls in flight must not write to a state that is gone (the engine may be gone already)
    delete s;
}

int zf_advance(zf_state *s, int32_t token) {
    if (!s) return fail(ZF_ERR_INVALID_ARG, "null argument");
    const zf_engine *e = s->eng;
    if (token < 0 || token >= e->V) return fail(ZF_ERR_RANGE, "token id out of range");
    const bool fresh = s->pending.empty();
    const int rc = feed_token_bytes(s, e->voc_bytes.data() + e->voc_off[token], e->voc_off[token + 1] - e->voc_off[token]);
    if (rc == ZF_OK && fresh && !s->pending.empty()) s->pending_token = token;   // the device will walk exactly this token from the state it knows
    return rc;
}

// Rows of a batch are independent (one state = one query).  A byte step of an ambiguous grammar
// costs O(set size squared) on the host, so a batch of wide charts is dealt to a few worker
// threads; batches of small charts (the common case: a pruned chart's sets hold a handful of
// items, Section 4.2) are fed by the caller's thread, where waking anybody would cost more than
// the work.
namespace {

struct AdvanceJob {
    zf_state *const *states;
    const int32_t *ids;          // null: the job is to bring the rows' charts up to date
    int32_t n;
    int32_t *rc;                 // [n]
    std::string *err;            // [n] the error text of a row that failed
    std::atomic<int32_t> next{0}, done{0};
};

int advance_one(zf_state *s, int32_t id) { return id < 0 ? zf_state_reset(s) : zf_advance(s, id); }

bool advance_rows(AdvanceJob &j) {   // takes rows until none is left; true if it fed any
    bool any = false;
    for (;;) {
        const int32_t b = j.next.fetch_add(1, std::memory_order_relaxed);
        if (b >= j.n) return any;
        if (j.ids) j.rc[b] = advance_one(j.states[b], j.ids[b]);
        else { (void)chart_of(j.states[b]); j.rc[b] = ZF_OK; }
        if (j.rc[b] != ZF_OK) j.err[b] = zf_last_error();   // the text lives in the worker's thread: hand it over
        j.done.fetch_add(1, std::memory_order_release);
        any = true;
    }
}

class AdvancePool {              // created on first use, never destroyed: its threads sleep until the process ends
  public:
    explicit AdvancePool(int n_workers) : n_workers_(n_workers), pid_(getpid()) {
        for (int i = 0; i < n_workers; i++) std::thread([this] { loop(); }).detach();
    }
    bool usable() const { return n_workers_ > 0 && pid_ == getpid(); }   // a forked child has the object but not the threads
    // The caller feeds rows too and returns when every row is done; a worker that wakes up late finds
    // no row left and never touches the caller's arrays (the job object itself is shared).
    void run(const std::shared_ptr<AdvanceJob> &j) {
        {
            std::lock_guard<std::mutex> lk(m_);
            job_ = j; epoch_++;
        }
        cv_work_.notify_all();
        advance_rows(*j);
        std::unique_lock<std::mutex> lk(m_);
        cv_done_.wait(lk, [&] { return j->done.load(std::memory_order_acquire) == j->n; });
        job_.reset();
    }

  private:
    void loop() {
        uint64_t seen = 0;
        for (;;) {
            std::shared_ptr<AdvanceJob> j;
            {
                std::unique_lock<std::mutex> lk(m_);
                cv_work_.wait(lk, [&] { return epoch_ != seen; });
                seen = epoch_;
                j = job_;
            }
            if (j && advance_rows(*j)) {
                { std::lock_guard<std::mutex> lk(m_); }     // the caller is either before its check or already waiting
                cv_done_.notify_one();
            }
        }
    }
    std::mutex m_;
    std::condition_variable cv_work_, cv_done_;
    std::shared_ptr<AdvanceJob> job_;
    uint64_t epoch_ = 0;
    int n_workers_ = 0;
    pid_t pid_;
};

std::mutex g_pool_mutex;         // one batch at a time through the pool; a second caller feeds its rows itself
AdvancePool *g_pool = nullptr;

// Host cost of feeding the rows' tokens, in item visits: Scan reads the current set once per byte,
// Complete of an ambiguous grammar pairs its items with each other, Compact sweeps the chart.
const int64_t ADVANCE_PARALLEL_FROM = 12000;   // about 0.1 ms of one core: below that the hand-over costs more than it saves
int64_t advance_cost(zf_state *const *states, const int32_t *ids, int32_t n) {
    int64_t cost = 0;
    for (int32_t b = 0; b < n; b++) {
        const zf_state *s = states[b];
        if (!s || ids[b] < 0 || ids[b] >= s->eng->V) continue;
        if (s->eng->host_aut) {
            // a walk through the host automaton costs nothing unless it meets a transition nobody has taken: then one Earley
            // byte step per byte from there on is the likely cost
            zf_engine *e = s->eng;
            std::lock_guard<std::mutex> rl(e->host_mu);
            const HostAutomaton &A = *e->host_aut;
            const bool placed = s->host_id == HostAutomaton::ROOT || s->host_id_epoch == e->host_epoch;
            if (placed && s->host_id == HostAutomaton::SINK) continue;
            const uint8_t first = e->voc_bytes[(size_t)e->voc_off[ids[b]]];
            const bool has_bytes = e->voc_off[ids[b] + 1] > e->voc_off[ids[b]];
            if (placed && has_bytes && A.st(s->host_id).trans[e->tab.cls[first]] != HostAutomaton::NONE) continue;
            const int64_t last = placed ? (int64_t)A.st(s->host_id).items.size() : 64, all = placed ? 8 * (int64_t)A.st(s->host_id).widest : 4096;
            cost += (e->voc_off[ids[b] + 1] - e->voc_off[ids[b]]) * (last + last * last / 16 + all);
            continue;
        }
        const Chart &c = chart_of(s);
        const int64_t last = c.set_off[c.n_sets()] - c.set_off[c.n_sets() - 1];
        cost += (s->eng->voc_off[ids[b] + 1] - s->eng->voc_off[ids[b]]) * (last + last * last / 16) + (int64_t)c.items.size();
    }
    return cost;
}

}  // namespace

// Bring the charts of a call's rows up to date (those fed through the host automaton lag behind): the same work as feeding
// them, so a batch of wide charts is dealt to the worker threads here as it is there.
static void catch_up_batch(zf_state *const *states, int32_t n) {
    int64_t cost = 0;
    int32_t lagging = 0;
    for (int32_t b = 0; b < n; b++) {
        const zf_state *s = states[b];
        if (!s || s->lag.empty()) continue;
        const Chart &c = s->chart;
        const int64_t last = c.set_off[c.n_sets()] - c.set_off[c.n_sets() - 1];
        cost += (int64_t)s->lag.size() * (last + last * last / 16) + (int64_t)c.items.size() * (int64_t)s->lag_cut.size();
        lagging++;
    }
    bool parallel = lagging >= 4 && cost >= ADVANCE_PARALLEL_FROM;
    if (parallel) {
        std::vector<const zf_state *> seen(states, states + n);
        std::sort(seen.begin(), seen.end());
        parallel = std::adjacent_find(seen.begin(), seen.end()) == seen.end();
    }
    std::unique_lock<std::mutex> pool_lock(g_pool_mutex, std::defer_lock);
    if (parallel) parallel = pool_lock.try_lock();
    if (parallel) {
        if (!g_pool) {
            const unsigned hw = std::thread::hardware_concurrency();
            g_pool = new AdvancePool((int)std::min(15u, std::max(1u, hw) - 1u));
        }
        parallel = g_pool->usable();
    }
    if (!parallel) {
        for (int32_t b = 0; b < n; b++) if (states[b]) (void)chart_of(states[b]);
        return;
    }
    std::vector<int32_t> rc((size_t)n, ZF_OK);
    std::vector<std::string> errs((size_t)n);
    auto job = std::make_shared<AdvanceJob>();
    job->states = states; job->ids = nullptr; job->n = n; job->rc = rc.data(); job->err = errs.data();
    g_pool->run(job);
}

int zf_advance_batch(zf_state *const *states, const int32_t *token_ids, int32_t n, int32_t *status) {
    if (!states || !token_ids || n < 0) return fail(ZF_ERR_INVALID_ARG, "null argument");
    for (int32_t b = 0; b < n; b++) if (!states[b]) return fail(ZF_ERR_INVALID_ARG, "null state");
    int first = ZF_OK;
    bool parallel = n >= 4 && advance_cost(states, token_ids, n) >= ADVANCE_PARALLEL_FROM;
    if (parallel) {                                       // every state at most once: a state named twice is fed twice, in order
        std::vector<const zf_state *> seen(states, states + n);
        std::sort(seen.begin(), seen.end());
        parallel = std::adjacent_find(seen.begin(), seen.end()) == seen.end();
    }
    std::unique_lock<std::mutex> pool_lock(g_pool_mutex, std::defer_lock);
    if (parallel) parallel = pool_lock.try_lock();
    if (parallel) {
        if (!g_pool) {
            const unsigned hw = std::thread::hardware_concurrency();
            g_pool = new AdvancePool((int)std::min(15u, std::max(1u, hw) - 1u));
        }
        parallel = g_pool->usable();
    }
    if (!parallel) {
        std::string first_err;
        for (int32_t b = 0; b < n; b++) {
            const int rc = advance_one(states[b], token_ids[b]);
            if (status) status[b] = rc;
            if (rc != ZF_OK && first == ZF_OK) { first = rc; first_err = zf_last_error(); }
        }
        if (first != ZF_OK) set_error(first_err);        // the caller sees the first failing row's text
        return first;
    }
    std::vector<int32_t> rc_store;
    if (!status) { rc_store.assign((size_t)n, ZF_OK); status = rc_store.data(); }
    std::vector<std::string> errs((size_t)n);
    auto job = std::make_shared<AdvanceJob>();
    job->states = states; job->ids = token_ids; job->n = n; job->rc = status; job->err = errs.data();
    g_pool->run(job);
    for (int32_t b = n - 1; b >= 0; b--)
        if (status[b] != ZF_OK) { first = status[b]; set_error(errs[b]); }
    return first;
}

int zf_advance_bytes(zf_state *s, const uint8_t *bytes, int64_t n) {
    if (!s || (n > 0 && !bytes) || n < 0) return fail(ZF_ERR_INVALID_ARG, "null argument");
    if (n == 0) return ZF_OK;
    return feed_token_bytes(s, bytes, n);
}

int zf_is_accepting(const zf_state *s, int32_t *out) {
    if (!s || !out) return fail(ZF_ERR_INVALID_ARG, "null argument");
    *out = s->accepting;
    return ZF_OK;
}

int zf_state_stats(const zf_state *s, zf_stats *o) {
    if (!s || !o) return fail(ZF_ERR_INVALID_ARG, "null argument");
    o->n_sets = chart_of(s).n_sets(); o->n_items = (int64_t)chart_of(s).items.size();
    o->items_created = s->items_created; o->bytes_fed = s->bytes_fed; o->accepting = s->accepting;
    return ZF_OK;
}

int zf_state_chart(const zf_state *s, int32_t *items, int64_t *set_off) {
    if (!s) return fail(ZF_ERR_INVALID_ARG, "null argument");
    if (items) for (size_t i = 0; i < chart_of(s).items.size(); i++) {
        items[3 * i] = chart_of(s).items[i].p; items[3 * i + 1] = (int32_t)chart_of(s).items[i].o; items[3 * i + 2] = chart_of(s).items[i].q;
    }
    if (set_off) for (size_t k = 0; k < chart_of(s).set_off.size(); k++) set_off[k] = chart_of(s).set_off[k];
    return ZF_OK;
}

int zf_position_info(const zf_engine *e, int32_t p, int32_t *lhs, int32_t *rule, int32_t *dot) {
    if (!e || p < 0 || p >= e->tab.P) return fail(ZF_ERR_INVALID_ARG, "bad position");
    if (lhs) *lhs = e->tab.pos_lhs_orig[p];
    if (rule) *rule = e->tab.pos_rule[p];
    if (dot) *dot = e->tab.pos_dot[p];
    return ZF_OK;
}

int zf_debug_host_mask(zf_engine *e, const zf_state *s, uint32_t *mask) { return zf_debug_host_mask_stats(e, s, mask, nullptr); }

int zf_debug_host_mask_cached(zf_engine *e, const zf_state *s, uint32_t *mask, int64_t *stats) {
    if (!e || !s || !mask || s->eng != e) return fail(ZF_ERR_INVALID_ARG, "bad argument");
    const Tables &t = e->tab;
    const Trie &tr = e->trie;
    Chart c = chart_of(s);
    const uint32_t m0 = c.n_sets();
    std::vector<uint32_t> ents(c.set_off[m0] - c.set_off[m0 - 1] + 1);
    const uint32_t n_ent = current_set_entries(t, c, ents.data());
    std::vector<uint32_t> valid(tr.Wr, 0), want(tr.Wr, 0);
    for (uint32_t k = 0; k < n_ent; k++)
        for (int w = 0; w < tr.Wr; w++) { valid[w] |= tr.ci_valid[(size_t)ents[k] * tr.Wr + w]; want[w] |= tr.ci_cd[(size_t)ents[k] * tr.Wr + w]; }
    for (int w = 0; w < tr.Wr; w++) want[w] &= ~valid[w];
    auto any_in = [&](uint32_t lo, uint32_t hi) { for (uint32_t r = lo; r < hi; r++) if ((want[r >> 5] >> (r & 31)) & 1) return true; return false; };
    int64_t n_steps = 0, n_wanted = 0, n_replay = 0, n_queued = 0;
    for (int w = 0; w < tr.Wr; w++) n_wanted += __builtin_popcount(want[w]);
    size_t chunk = 0;
    int64_t last_counted = -1;
    for (uint32_t i = 0; i < tr.nodes.size();) {
        const TrieNode &nd = tr.nodes[i];
        if (!any_in(nd.rank, nd.rank + nd.n_sub)) { i = nd.skip; continue; }
        while (chunk + 1 < tr.chunk_begin.size() && tr.chunk_end[chunk] <= i) chunk++;
        if ((int64_t)chunk != last_counted) {    // the kernel walks chunk by chunk and replays the path above each chunk's first node
            last_counted = (int64_t)chunk; n_queued++;
            n_replay += tr.nodes[tr.chunk_begin[chunk]].depth - 1;
        }
        c.truncate(m0 + nd.depth - 1);
        StepResult r = earley_step(t, c, nd.byte, false, nullptr);
        n_steps++;
        if (nd.has_string && r.alive && ((want[nd.rank >> 5] >> (nd.rank & 31)) & 1)) valid[nd.rank >> 5] |= 1u << (nd.rank & 31);
        i = r.kernel_nonempty ? i + 1 : nd.skip;
    }
    memset(mask, 0, sizeof(uint32_t) * e->W);
    for (int v = 0; v < e->V; v++) {
        uint32_t r = tr.rank_of[v];
        if (r != 0xFFFFFFFFu && ((valid[r >> 5] >> (r & 31)) & 1)) mask[v >> 5] |= 1u << (v & 31);
    }
    if (stats) { stats[0] = n_steps; stats[1] = n_wanted; stats[2] = n_ent; stats[3] = n_replay; stats[4] = n_queued; }
    return ZF_OK;
}

int zf_debug_host_mask_stats(zf_engine *e, const zf_state *s, uint32_t *mask, int64_t *stats) {
    if (!e || !s || !mask || s->eng != e) return fail(ZF_ERR_INVALID_ARG, "bad argument");
    int64_t n_steps = 0, n_alive = 0, max_path = 0, max_set = 0, chunks_over = 0;
    const int CHUNK_RANKS = e->trie.chunk_ranks;
    std::vector<uint8_t> chunk_over((e->trie.n_strings + CHUNK_RANKS - 1) / CHUNK_RANKS + 1, 0);
    const Tables &t = e->tab;
    const Trie &tr = e->trie;
    Chart c = chart_of(s);
    const uint32_t m0 = c.n_sets();
    std::vector<uint8_t> ok(tr.n_strings, 0);
    for (uint32_t i = 0; i < tr.nodes.size();) {
        const TrieNode &nd = tr.nodes[i];
        c.truncate(m0 + nd.depth - 1);
        StepResult r = earley_step(t, c, nd.byte, false, nullptr);
        if (nd.has_string && r.alive) ok[nd.rank] = 1;
        n_steps++; n_alive += r.alive;
        int64_t path = (int64_t)c.items.size() - c.set_off[m0];
        int64_t last = (int64_t)c.items.size() - c.set_off[c.n_sets() - 1];
        if (path > max_path) max_path = path;
        if (last > max_set) max_set = last;
        if (path > e->opt.lane_item_cap && !chunk_over[nd.rank / CHUNK_RANKS]) { chunk_over[nd.rank / CHUNK_RANKS] = 1; chunks_over++; }
        i = r.kernel_nonempty ? i + 1 : nd.skip;
    }
    if (stats) { stats[0] = n_steps; stats[1] = n_alive; stats[2] = max_path; stats[3] = max_set; stats[4] = chunks_over; }
    memset(mask, 0, sizeof(uint32_t) * e->W);
    for (int v = 0; v < e->V; v++) {
        uint32_t r = tr.rank_of[v];
        if (r != 0xFFFFFFFFu && ok[r]) mask[v >> 5] |= 1u << (v & 31);
    }
    return ZF_OK;
}

// The packed form of a chart: [n_sets][set offsets][item word, origin]...; what the kernels read, and the state cache's key.
static void pack_chart(const Tables &t, const Chart &c, std::vector<uint32_t> &k) {
    k.clear();
    k.push_back(c.n_sets());
    k.insert(k.end(), c.set_off.begin(), c.set_off.end());
    for (const Item &it : c.items) {   // host item -> device item word + origin
        const uint32_t aw = t.advpq[it.p];
        k.push_back((aw & IW_TERM) ? ((aw & 0xFFFFu) | ((uint32_t)it.q << 16)) : aw);
        k.push_back(it.o);
    }
}

// State cache (Section 5.2): find every row's pool slot by its packed chart; rows seen for the first time get a slot
// (round-robin victim, never one handed out in the same call) and are listed in miss_rows.  Returns the number of hits.
static int state_cache_lookup(DeviceSide *d, const std::vector<std::vector<uint32_t>> &packed, int32_t batch,
                              std::vector<uint32_t> &row_slot, std::vector<uint32_t> &miss_rows) {
    int n_hits = 0;
    const uint32_t call = ++d->cache_call;
    for (int b = 0; b < batch; b++) {
        const std::vector<uint32_t> &k = packed[b];
        uint64_t h = 0xCBF29CE484222325ull;
        for (uint32_t w : k) { h ^= w; h *= 0x100000001B3ull; h ^= h >> 29; }
        uint32_t found = 0xFFFFFFFFu;
        auto range = d->cache_index.equal_range(h);
        for (auto it = range.first; it != range.second; ++it) if (d->cache[it->second].key == k) { found = it->second; break; }
        if (found == 0xFFFFFFFFu) {
            while (d->cache[d->cache_victim].used && d->cache[d->cache_victim].stamp == call) d->cache_victim = (d->cache_victim + 1) % d->cache.size();
            found = d->cache_victim;
            d->cache_victim = (d->cache_victim + 1) % d->cache.size();
            DeviceSide::CacheEntry &ce = d->cache[found];
            if (ce.used) {   // evict
                auto r2 = d->cache_index.equal_range(ce.hash);
                for (auto it = r2.first; it != r2.second; ++it) if (it->second == found) { d->cache_index.erase(it); break; }
            }
            ce.hash = h; ce.key = k; ce.used = true;
            d->cache_index.emplace(h, found);
            miss_rows.push_back((uint32_t)b);
        } else n_hits++;
        d->cache[found].stamp = call;
        row_slot[b] = found;
    }
    return n_hits;
}

static int enqueue_store_impl(zf_engine *e, zf_state *const *states, int32_t batch, uint32_t *d_mask, void *hip_stream, bool wait, uint32_t slot);
// zf_compute_mask_apply_async: the logits the call's mask is to be applied to.  The mask kernel over the persistent automaton
// takes them along when it can (fused = true); whoever set the request launches the logit-masking kernel otherwise.
struct ApplyRequest { const void *logits = nullptr; void *out = nullptr; int64_t stride = 0; int32_t dtype = 0; bool fused = false; };
static thread_local ApplyRequest g_apply;

// Pack and upload the charts and enqueue the kernels of one compute_mask call: upload, mask kernel,
// closing kernel (fallback pass for what the mask kernel listed + permutation into token order),
// gather when the state cache is on.  wait = true: also wait and return the final status.
// noalloc = true (zf_compute_mask_noalloc): every per-call device buffer is a slice of the device's static scratch array,
// the state cache is passed by, and a call that does not fit the array or the staging room is refused.
static int enqueue_mask_impl(zf_engine *e, zf_state *const *states, int32_t batch, uint32_t *d_mask, void *hip_stream, bool wait, bool noalloc, bool per_block) {
    if (!e || !states || batch <= 0 || batch > MAX_BATCH || !d_mask) return fail(ZF_ERR_INVALID_ARG, "bad argument (batch must be 1..4096)");
    DeviceSide *d = e->dev;
    if (!d) return fail(ZF_ERR_DEVICE, "engine was compiled without a device (device = -1)");
    hipStream_t stream = (hipStream_t)hip_stream;
    HIP_TRY(hipSetDevice(d->device));
    if (d->pending >= (uint32_t)DeviceSide::N_SLOTS) return fail(ZF_ERR_INVALID_ARG, "too many asynchronous mask calls in flight: call zf_mask_wait");
    const uint32_t slot = d->next_slot;
    if (d->pending) HIP_TRY(hipEventSynchronize(d->stage_done[slot]));   // the slot's previous upload has left the staging buffer (with no call in flight zf_mask_wait has seen to that)
    for (int b = 0; b < batch; b++)
        if (!states[b] || states[b]->eng != e) return fail(ZF_ERR_INVALID_ARG, "state " + std::to_string(b) + " is null or belongs to another engine");
    if (e->store_on && !noalloc && !per_block) return enqueue_store_impl(e, states, batch, d_mask, hip_stream, wait, slot);
    catch_up_batch(states, batch);                        // these paths send the charts
    // ---- the packed form of every row: [n_sets][set offsets][item word, origin]... (also the cache key) ----
    static thread_local std::vector<std::vector<uint32_t>> packed;
    if ((int)packed.size() < batch) packed.resize(batch);
    for (int b = 0; b < batch; b++) pack_chart(e->tab, chart_of(states[b]), packed[b]);
    // ---- state cache: rows whose chart has been seen before only need their finished mask copied ----
    const bool sc = !noalloc && !d->cache.empty() && (size_t)batch * 2 <= d->cache.size();
    static thread_local std::vector<uint32_t> row_slot, miss_rows;
    row_slot.assign(batch, 0);
    miss_rows.clear();
    int n_hits = 0;
    if (sc) n_hits = state_cache_lookup(d, packed, batch, row_slot, miss_rows);
    else for (int b = 0; b < batch; b++) miss_rows.push_back((uint32_t)b);
    // trie walk: rows with a wide current set first: their chunks are the expensive ones, and work that starts early does
    // not end up as the kernel's tail (the mask automaton gives every row its own blocks: the order does not matter there)
    if (e->opt.walk_mode == 1) std::stable_sort(miss_rows.begin(), miss_rows.end(), [&](uint32_t x, uint32_t y) {
        const Chart &cx = chart_of(states[x]), &cy = chart_of(states[y]);
        return cx.set_off[cx.n_sets()] - cx.set_off[cx.n_sets() - 1] > cy.set_off[cy.n_sets()] - cy.set_off[cy.n_sets() - 1];
    });
    const int nb = (int)miss_rows.size();                // rows that go through the kernels
    d->report.cache_hits = n_hits; d->report.cache_misses = sc ? nb : 0;
    // ---- upload: [RowChart x nb][set offsets][items][cache rows of the token-mask cache][dst slot x nb][row slot x batch] ----
    size_t n_off = 0, n_items = 0, n_ent = 0, max_off = 0, max_items = 0, max_ent = 0;
    const bool use_cache = !e->opt.disable_token_mask_cache;
    for (int r = 0; r < nb; r++) {
        const Chart &c = chart_of(states[miss_rows[r]]);
        const size_t last = c.set_off[c.n_sets()] - c.set_off[c.n_sets() - 1];
        n_off += c.set_off.size();
        n_items += c.items.size();
        if (use_cache) n_ent += last;
        max_off = std::max(max_off, c.set_off.size()); max_items = std::max(max_items, c.items.size());
        if (use_cache) max_ent = std::max(max_ent, last);
    }
    // Mask automaton: when the rows' charts are of similar size each row's sections get the same room, so that a block
    // can request its row's sets, items and cache rows without waiting for the row's header (one memory round trip
    // instead of two; the round trip is over PCIe when the kernels read the staging slot directly).
    const bool uniform = e->opt.walk_mode != 1 && nb > 0 &&
                         (size_t)nb * (4 * max_off + 8 * max_items + 4 * max_ent) <= 2 * (4 * n_off + 8 * n_items + 4 * n_ent) + 4096;
    if (uniform) { n_off = (size_t)nb * max_off; n_items = (size_t)nb * max_items; n_ent = (size_t)nb * max_ent; }
    auto align16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
    const size_t off_rows = 0, off_so = align16(sizeof(RowChart) * nb), off_items = align16(off_so + 4 * n_off);
    const size_t off_ent = align16(off_items + sizeof(Item) * n_items);
    const size_t off_dst = align16(off_ent + 4 * n_ent), off_rowslot = align16(off_dst + 4 * (size_t)nb);
    const size_t total = off_rowslot + 4 * (size_t)batch + 16;
    if (noalloc && total > d->stage_cap[slot])
        return fail(ZF_ERR_INVALID_ARG, "zf_compute_mask_noalloc: the packed charts (" + std::to_string(total) + " bytes) exceed the staging room of " +
                                        std::to_string(d->stage_cap[slot]) + " bytes");
    if (total > d->stage_cap[slot]) {
        if (d->h_stage[slot]) (void)hipHostFree(d->h_stage[slot]);
        d->h_stage[slot] = nullptr; d->stage_cap[slot] = 0;
        size_t cap = total * 2 + 4096;
        HIP_TRY(hipHostMalloc(&d->h_stage[slot], cap, hipHostMallocDefault));
        d->stage_cap[slot] = cap;
    }
    if (!noalloc && total > d->chart_cap) {
        HIP_TRY(hipStreamSynchronize(stream));            // earlier calls may still read the old buffer
        if (d->d_chart) (void)hipFree(d->d_chart);
        d->d_chart = nullptr; d->chart_cap = 0;
        size_t cap = total * 2 + 4096;
        HIP_TRY(hipMalloc(&d->d_chart, cap));
        d->chart_cap = cap;
    }
    uint32_t n_cache_rows = 0;                            // distinct rows of the token-mask cache, summed over the rows of the call
    {
        uint8_t *h = (uint8_t *)d->h_stage[slot];
        RowChart *rows = (RowChart *)(h + off_rows);
        uint32_t *so = (uint32_t *)(h + off_so);
        uint32_t *dev_items = (uint32_t *)(h + off_items);
        uint32_t *ents = (uint32_t *)(h + off_ent);
        uint32_t *dst = (uint32_t *)(h + off_dst);
        memcpy(h + off_rowslot, row_slot.data(), 4 * (size_t)batch);
        uint32_t so_at = 0, it_at = 0, en_at = 0;
        for (int r = 0; r < nb; r++) {
            const Chart &c = chart_of(states[miss_rows[r]]);
            const std::vector<uint32_t> &k = packed[miss_rows[r]];
            if (uniform) { so_at = (uint32_t)(r * max_off); it_at = (uint32_t)(r * max_items); en_at = (uint32_t)(r * max_ent); }
            rows[r] = RowChart{c.n_sets(), so_at, it_at, en_at, 0, (uint32_t)c.items.size(), {0, 0}};
            if (use_cache) rows[r].n_ent = current_set_entries(e->tab, c, ents + en_at);
            n_cache_rows += rows[r].n_ent;
            en_at += rows[r].n_ent;
            memcpy(so + so_at, k.data() + 1, 4 * c.set_off.size());
            memcpy(dev_items + 2 * (size_t)it_at, k.data() + 1 + c.set_off.size(), 8 * c.items.size());
            so_at += (uint32_t)c.set_off.size(); it_at += (uint32_t)c.items.size();
            dst[r] = sc ? row_slot[miss_rows[r]] : miss_rows[r];
        }
    }
    // ---- per-call device buffers ----
    const size_t need_rank = (size_t)std::max(nb, 1) * d->tab.Wr, need_ovf = 2 * (size_t)std::max(nb, 1) * d->tab.n_chunks;   // the automaton kernel may name a chunk in two entries
    // zf_compute_mask_noalloc: the same buffers as slices of the static array: [counters: 64 words][fallback set starts][fallback
    // arenas][rank-ordered verdict words][device copy of the charts (trie walk)][the trie walk's queue][fallback list: what is left]
    uint8_t *const scr = d->scratch;
    size_t scr_ss = 0, scr_fb = 0, scr_rank = 0, scr_chart = 0, scr_work = 0, scr_ovf = 0, scr_ovf_cap = 0;
    if (noalloc) {
        auto align256 = [](size_t x) { return (x + 255) & ~(size_t)255; };
        scr_ss = 1024;
        scr_fb = align256(scr_ss + (size_t)(FB_DEPTH_MAX + 2) * NOALLOC_FB_WAVES * 4);
        scr_rank = align256(scr_fb + (size_t)NOALLOC_FB_WAVES * NOALLOC_FB_ITEMS_PER_WAVE * sizeof(uint2));
        scr_chart = align256(scr_rank + need_rank * 4 + 16);
        scr_work = align256(scr_chart + (e->opt.walk_mode == 1 ? total + 16 : 0));
        scr_ovf = align256(scr_work + (e->opt.walk_mode == 1 ? (size_t)std::max(nb, 1) * d->tab.n_chunks * sizeof(uint4) + 16 : 0));
        if (scr_ovf + 4096 * sizeof(uint4) > NOALLOC_SCRATCH_BYTES)
            return fail(ZF_ERR_INVALID_ARG, "zf_compute_mask_noalloc: batch x vocabulary needs " + std::to_string(scr_ovf + 4096 * sizeof(uint4)) +
                                            " bytes of scratch memory, the static array holds " + std::to_string(NOALLOC_SCRATCH_BYTES));
        scr_ovf_cap = std::min(need_ovf, (NOALLOC_SCRATCH_BYTES - scr_ovf) / sizeof(uint4));   // a longer list fails the call loudly (ZF_ERR_OVERFLOW)
    } else if (need_rank > d->rank_cap || need_ovf > d->overflow_cap) {
        HIP_TRY(hipStreamSynchronize(stream));
        if (d->d_rank_mask) (void)hipFree(d->d_rank_mask);
        if (d->d_overflow) (void)hipFree(d->d_overflow);
        if (d->d_work) (void)hipFree(d->d_work);
        d->d_rank_mask = nullptr; d->d_overflow = nullptr; d->d_work = nullptr; d->rank_cap = d->overflow_cap = 0;
        HIP_TRY(hipMalloc((void **)&d->d_rank_mask, need_rank * 4 + 16));
        HIP_TRY(hipMalloc((void **)&d->d_overflow, need_ovf * sizeof(uint4) + 16));
        HIP_TRY(hipMalloc((void **)&d->d_work, need_ovf * sizeof(uint4) + 16));
        d->rank_cap = need_rank; d->overflow_cap = need_ovf;
    }
    MaskArgs a{};
    a.tab = d->tab;
    // Where the kernels read the packed charts: with the mask automaton and the state cache off, straight from the pinned
    // staging slot (a block needs a few hundred bytes once; the copy to device memory would be a kernel of its own at the
    // head of the call); else from the device copy that upload_kernel makes.
    const bool direct = e->opt.walk_mode != 1 && !sc;
    uint8_t *chart_base = direct ? (uint8_t *)d->h_stage[slot] : (noalloc ? scr + scr_chart : (uint8_t *)d->d_chart);
    a.rows = (const RowChart *)(chart_base + off_rows);
    a.set_off = (const uint32_t *)(chart_base + off_so);
    a.items = (const Item *)(chart_base + off_items);
    a.entries = (const uint32_t *)(chart_base + off_ent);
    a.rank_mask = noalloc ? (uint32_t *)(scr + scr_rank) : d->d_rank_mask;
    a.out_mask = sc ? d->d_pool : d_mask;                 // with the state cache the rows are finished in their pool slots
    a.dst_row = direct ? nullptr : (const uint32_t *)(chart_base + off_dst);   // null: row r of the launch is row r of the output (no state cache: every row runs)
    a.row_slot = (const uint32_t *)(chart_base + off_rowslot);
    a.so_stride = uniform ? (uint32_t)max_off : 0u; a.it_stride = uniform ? (uint32_t)max_items : 0u; a.ent_stride = uniform ? (uint32_t)max_ent : 0u;
    a.user_mask = d_mask;
    a.user_batch = batch;
    a.handoff_in_permute = sc ? 0 : 1;
    if (noalloc) {                                        // cleared at the head of the call; counters_next is a spare set
        a.counters = (uint32_t *)scr; a.counters_next = (uint32_t *)scr + COUNTER_SET_WORDS;
    } else {
        a.counters = d->d_counters + COUNTER_SET_WORDS * d->call_parity;
        a.counters_next = d->d_counters + COUNTER_SET_WORDS * (d->call_parity ^ 1u);
        d->call_parity ^= 1u;
    }
    a.work = noalloc ? (uint4 *)(scr + scr_work) : d->d_work;
    a.host_status = d->h_status + 8 * slot;
    if (++d->call_seq == 0) d->call_seq = 1;
    a.seq = d->call_seq;
    a.overflow_list = noalloc ? (uint4 *)(scr + scr_ovf) : d->d_overflow;
    a.overflow_cap = (uint32_t)(noalloc ? scr_ovf_cap : d->overflow_cap);
    a.fb_items = noalloc ? (uint2 *)(scr + scr_fb) : d->d_fb_items;
    a.fb_set_start = noalloc ? (uint32_t *)(scr + scr_ss) : d->d_fb_ss;
    a.fb_waves = noalloc ? NOALLOC_FB_WAVES : FB_WAVES;
    a.fb_stride = noalloc ? NOALLOC_FB_ITEMS_PER_WAVE : FB_ITEMS_PER_WAVE;
    a.batch = nb;
    // Item budget of a walking wavefront: the configured one, raised for this call when the rows'
    // current sets are large (ambiguous grammars) so that such rows do not all end in the fallback.
    a.lane_cap = e->opt.lane_item_cap;
    if (e->lane_cap_auto) {
        size_t widest = 0;
        for (int r = 0; r < nb; r++) {
            const Chart &c = chart_of(states[miss_rows[r]]);
            widest = std::max<size_t>(widest, c.set_off[c.n_sets()] - c.set_off[c.n_sets() - 1]);
        }
        size_t want_cap = (8 * widest + 64 + 31) / 32 * 32;
        while (want_cap > (size_t)a.lane_cap && walk_lds_bytes(d->tab, d->mode, (int)std::min<size_t>(want_cap, LANE_CAP_MAX)) > 160u * 1024u) want_cap -= 32;
        if (want_cap > (size_t)a.lane_cap) a.lane_cap = (int)std::min<size_t>(want_cap, LANE_CAP_MAX);
    }
    {   // the persistent walk grid: as many blocks as the chip holds at once (LDS is the limit)
        const uint32_t lds = walk_lds_bytes(d->tab, d->mode, a.lane_cap);
        if (lds != d->occ_lds) {                          // ask the runtime once per LDS size
            HIP_TRY(walk_blocks_per_cu(d->mode, lds, &d->occ_blocks));
            d->occ_lds = lds;
        }
        // half as many blocks again as the chip holds at once: the surplus blocks take the places of
        // blocks whose share of the queue was light (measured: exactly-resident grids are ~10 % slower,
        // larger surpluses bring nothing more)
        a.walk_blocks = std::max(1, d->cus) * d->occ_blocks * 3 / 2;
    }
    a.fb_cap = (int32_t)std::min<uint32_t>((uint32_t)e->opt.fallback_item_cap, a.fb_stride);
    a.mode = d->mode;
    const bool automaton = e->opt.walk_mode != 1;
    if (automaton) {
        // LDS budgets of one block's automaton.  The set under construction gets the configured item
        // budget (tests set it tiny to force the fallback pass), else room for sets a few times as wide
        // as the widest current set; states and the item arena share what the tables leave of 160 KB.
        size_t widest = 0, most_sets = 0, most_items = 0, biggest_set = 0;
        for (int r = 0; r < nb; r++) {
            const Chart &c = chart_of(states[miss_rows[r]]);
            widest = std::max<size_t>(widest, c.set_off[c.n_sets()] - c.set_off[c.n_sets() - 1]);
            most_sets = std::max<size_t>(most_sets, c.n_sets());
            most_items = std::max<size_t>(most_items, c.set_off[c.n_sets()]);
            for (uint32_t k = 0; k < c.n_sets(); k++) biggest_set = std::max<size_t>(biggest_set, c.set_off[k + 1] - c.set_off[k]);
        }
        int scratch = 0, n_states = 0, arena = 0, base_sets = 0, base_items = 0;
        // The build without the wide byte step also takes the chart from LDS only (its pointers are then
        // known to be LDS addresses): it serves calls whose sets are all small and whose charts all fit.
        bool wide = biggest_set > (size_t)AUT_NARROW_SET_MAX;
        const uint32_t lds_max = 160u * 1024u;
        for (;;) {
            scratch = e->lane_cap_auto ? (int)std::min<size_t>(LANE_CAP_MAX, (4 * widest + 128 + 31) / 32 * 32) : e->opt.lane_item_cap;
            n_states = AUT_STATES_DEFAULT; arena = std::max(1024, 8 * scratch);
            base_sets = BASE_SETS_LDS; base_items = BASE_ITEMS_LDS;
            auto lds_now = [&]() { return automaton_lds_bytes(d->tab, d->mode, n_states, arena, scratch, base_sets, base_items, wide); };
            while (lds_now() > lds_max && arena > 2 * scratch) arena /= 2;
            while (lds_now() > lds_max && n_states > 8) n_states /= 2;
            while (lds_now() > lds_max && scratch > 32) { scratch /= 2; arena = std::max(arena / 2, 2 * scratch); }
            if (lds_now() > lds_max) return fail(ZF_ERR_INVALID_ARG, "the grammar tables leave no LDS for the mask automaton");
            // the rows' charts are read over and over by Complete: keep them in LDS too when the longest one fits in what is left
            if (most_sets > (size_t)BASE_SETS_LDS || most_items > (size_t)BASE_ITEMS_LDS) {
                const int want_sets = (int)std::max<size_t>(BASE_SETS_LDS, (most_sets + 32) / 32 * 32 - 1);
                const int want_items = (int)std::max<size_t>(BASE_ITEMS_LDS, (most_items + 63) / 64 * 64);
                if (want_sets <= AUT_BASE_SETS_MAX && want_items <= AUT_BASE_ITEMS_MAX &&
                    automaton_lds_bytes(d->tab, d->mode, n_states, arena, scratch, want_sets, want_items, wide) <= lds_max) {
                    base_sets = want_sets; base_items = want_items;
                }
            }
            if (wide || (most_sets <= (size_t)base_sets && most_items <= (size_t)base_items)) break;
            wide = true;                                  // some chart stays in global memory: the other build
        }
        a.aut_states = n_states; a.aut_arena = arena; a.aut_scratch = scratch;
        a.aut_base_sets = base_sets; a.aut_base_items = base_items;
        a.aut_wide = wide ? 1 : 0;
        // blocks per row: enough to fill the chip about once, at most one block per pass of AUT_SUB_WORDS words
        const int n_sub = (d->tab.Wr + AUT_SUB_WORDS - 1) / AUT_SUB_WORDS;
        a.aut_parts = std::max(1, std::min(n_sub, (2 * std::max(1, d->cus) + std::max(nb, 1) - 1) / std::max(nb, 1)));
    }
    const bool prof = d->profiling;
    d->report.chart_bytes = (int64_t)total;
    d->report.cache_rows = (int32_t)n_cache_rows;
    d->report.main_ms = d->report.fallback_ms = d->report.permute_ms = 0.f;
    d->report.overflow_chunks = d->report.walk_chunks = d->report.parser_steps = 0;
    // everything the host has to work out is done: enqueue the upload and the kernels back to back
    if (noalloc) HIP_TRY(launch_clear_words((uint32_t *)scr, 2 * COUNTER_SET_WORDS, stream));   // the array keeps the last call's counters
    if (!direct) HIP_TRY(launch_upload(d->h_stage[slot], chart_base, total, stream));
    const bool run_kernels = nb > 0;
    if (run_kernels && d->tab.n_chunks > 0 && !automaton) HIP_TRY(launch_cache_merge(a, stream));
    if (prof) HIP_TRY(hipEventRecord(d->ev[0], stream));
    if (run_kernels && d->tab.n_chunks > 0) HIP_TRY(automaton ? launch_mask_automaton(a, stream) : launch_mask_walk(a, stream));
    if (prof) HIP_TRY(hipEventRecord(d->ev[1], stream));
    d->closing_kernel = true;
    if (run_kernels) HIP_TRY(launch_finish(a, d->cus, stream));   // fallback pass (if anything was listed) + permutation; also hands the counters to the host and clears the next call's
    if (sc) HIP_TRY(launch_gather(a, stream));            // every row's finished mask from its pool slot to the caller's tensor
    if (prof) HIP_TRY(hipEventRecord(d->ev[3], stream));
    HIP_TRY(hipEventRecord(d->stage_done[slot], stream));   // the staging slot is free again once this point of the stream is reached
    d->next_slot = (slot + 1) % DeviceSide::N_SLOTS;
    d->pending++;
    d->last_seq = a.seq; d->last_slot = slot;
    if (!wait) return ZF_OK;
    HIP_TRY(hipStreamSynchronize(stream));               // the waiting call returns with the mask complete, not only its status known
    return zf_mask_wait(e, hip_stream);
}

// The same call through the persistent automaton (walk_mode 2): the upload names, per row, the state the row was last known
// to be in and the byte classes fed since; the mask kernel walks them, checks the vocabulary from the state it arrives at and
// reports that state back (pinned memory), which zf_mask_wait notes in the zf_state.  Rows the store does not know -- after it
// was cleared, or too far behind -- bring their packed chart along and are made states of by the import kernel first.
// The state's name in the host automaton, when it has a current one there (the caller holds the host automaton's lock) ...
static bool host_name_valid(const zf_engine *e, const zf_state *st) {
    return e->host_aut && st->host_id != HostAutomaton::ROOT && st->host_id_epoch == e->host_epoch && st->host_id < HostAutomaton::SINK && st->host_id != 0;
}
// ... and the device's name of that state, 0 when the device has not reported one
static uint32_t device_name_of(const zf_engine *e, const zf_state *st) {
    return host_name_valid(e, st) ? e->dev->name_find(st->host_id, e->host_epoch, e->dev->store_epoch) : 0u;
}

static int enqueue_store_impl(zf_engine *e, zf_state *const *states, int32_t batch, uint32_t *d_mask, void *hip_stream, bool wait, uint32_t slot) {
    DeviceSide *d = e->dev;
    hipStream_t stream = (hipStream_t)hip_stream;
    std::unique_lock<std::mutex> host_lk;                 // the rows' current sets are read from the host automaton (a row it does not know is brought in)
    if (e->host_aut) host_lk = std::unique_lock<std::mutex>(e->host_mu);
    // ---- clear the store when it is new, half full, or has refused a request; only with no call in flight ----
    if (d->pending == 0 && (d->store_dirty || d->store_states > d->store.cap_states / 2 || d->store_items > d->store.cap_items / 2)) {
        HIP_TRY(launch_store_clear(d->store, (uint32_t)std::max(e->tab.n_cls, 1), d->d_root_items, d->n_root, stream));
        d->store_epoch++;
        d->store_states = 2; d->store_items = d->n_root;
        d->store_dirty = false;
    }
    // ---- state cache (keyed by the packed chart, as on the other paths) ----
    const bool sc = !d->cache.empty() && (size_t)batch * 2 <= d->cache.size();
    static thread_local std::vector<std::vector<uint32_t>> packed;
    static thread_local std::vector<uint32_t> row_slot, miss_rows, import_rows;
    if ((int)packed.size() < batch) packed.resize(batch);
    row_slot.assign(batch, 0);
    miss_rows.clear();
    int n_hits = 0;
    if (sc) {
        catch_up_batch(states, batch);                    // the state cache's key is the packed chart
        for (int b = 0; b < batch; b++) pack_chart(e->tab, chart_of(states[b]), packed[b]);
        n_hits = state_cache_lookup(d, packed, batch, row_slot, miss_rows);
    } else {
        for (int b = 0; b < batch; b++) miss_rows.push_back((uint32_t)b);
        // rows the store does not know come in through their charts (all of them after the store was cleared)
        static thread_local std::vector<zf_state *> unknown;
        unknown.clear();
        for (int b = 0; b < batch; b++) {
            zf_state *st = states[b];
            if (st->dev_id == STORE_ROOT_ID || (st->dev_id != 0 && st->dev_epoch == d->store_epoch) || st->lag.empty()) continue;
            if (device_name_of(e, st)) continue;          // the device knows the state under the name the host automaton has for it: no chart needed
            unknown.push_back(st);
        }
        if (!unknown.empty()) catch_up_batch(unknown.data(), (int32_t)unknown.size());
    }
    const int nb = (int)miss_rows.size();
    d->report.cache_hits = n_hits; d->report.cache_misses = sc ? nb : 0;
    // ---- what each launched row sends ----
    import_rows.clear();
    static thread_local std::vector<uint32_t> row_named;  // per launched row: the device's name of the state it stands in, when the host automaton's name for it has one (0: not known)
    row_named.assign(miss_rows.size(), 0);
    const bool use_cache = !e->opt.disable_token_mask_cache;
    size_t n_pend = 0, n_ent = 0, n_off = 0, n_items = 0, widest = 0, biggest_set = 0;
    for (int r = 0; r < nb; r++) {
        zf_state *st = states[miss_rows[r]];
        const CurrentSet cs = current_set(st);
        const size_t last = cs.n;
        widest = std::max(widest, last);
        biggest_set = std::max<size_t>(biggest_set, cs.biggest);
        if (use_cache) n_ent += last;
        row_named[r] = device_name_of(e, st);
        const bool known = st->dev_id == STORE_ROOT_ID || (st->dev_id != 0 && st->dev_epoch == d->store_epoch);
        if (row_named[r]) {}                               // sent with its name on the device: no bytes, no chart
        else if (known) n_pend += st->pending.size();
        else {
            const Chart &c = chart_of(st);
            import_rows.push_back((uint32_t)r);
            if (!sc) pack_chart(e->tab, c, packed[miss_rows[r]]);
            n_off += c.set_off.size(); n_items += c.items.size();
        }
    }
    const int n_imp = (int)import_rows.size();
    auto align16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
    const size_t off_srow = 0, off_ent = align16(sizeof(StoreRow) * nb), off_pend = align16(off_ent + 4 * n_ent);
    const size_t off_dst = align16(off_pend + n_pend), off_rowslot = align16(off_dst + 4 * (size_t)nb);
    const size_t off_rows = align16(off_rowslot + 4 * (size_t)batch), off_so = align16(off_rows + sizeof(RowChart) * n_imp);
    const size_t off_items = align16(off_so + 4 * n_off), off_imp = align16(off_items + sizeof(Item) * n_items);
    const size_t total = off_imp + 4 * (size_t)n_imp + 16;
    if (total > d->stage_cap[slot]) {
        if (d->h_stage[slot]) (void)hipHostFree(d->h_stage[slot]);
        d->h_stage[slot] = nullptr; d->stage_cap[slot] = 0;
        const size_t cap = total * 2 + 4096;
        HIP_TRY(hipHostMalloc(&d->h_stage[slot], cap, hipHostMallocDefault));
        d->stage_cap[slot] = cap;
    }
    if (sc && total > d->chart_cap) {
        HIP_TRY(hipStreamSynchronize(stream));
        if (d->d_chart) (void)hipFree(d->d_chart);
        d->d_chart = nullptr; d->chart_cap = 0;
        const size_t cap = total * 2 + 4096;
        HIP_TRY(hipMalloc(&d->d_chart, cap));
        d->chart_cap = cap;
    }
    DeviceSide::CallRecord &rec = d->rec[slot];
    rec.active = true; rec.epoch = d->store_epoch;
    rec.st.assign(nb, std::shared_ptr<StateLink>()); rec.gen.assign(nb, 0); rec.upto.assign(nb, 0); rec.hop.assign(nb, 0);
    rec.host.assign(nb, 0); rec.host_epoch = e->host_epoch;
    if (d->hop_epoch != d->store_epoch) { if (d->hop_used) std::fill(d->hop_key.begin(), d->hop_key.end(), 0); d->hop_used = 0; d->hop_epoch = d->store_epoch; }
    uint32_t n_cache_rows = 0;
    static thread_local std::vector<uint32_t> row_n_ent, row_ent_at, row_n_items;
    row_n_ent.assign(nb, 0); row_ent_at.assign(nb, 0); row_n_items.assign(nb, 0);
    static thread_local StoreMiniRows mini;               // short records: they travel in the kernel's argument block
    const bool use_mini = nb <= STORE_MINI_ROWS;
    {
        uint8_t *h = (uint8_t *)d->h_stage[slot];
        StoreRow *srow = (StoreRow *)(h + off_srow);
        uint32_t *ents = (uint32_t *)(h + off_ent);
        uint8_t *pend = h + off_pend;
        uint32_t *dst = (uint32_t *)(h + off_dst);
        RowChart *rows = (RowChart *)(h + off_rows);
        uint32_t *so = (uint32_t *)(h + off_so);
        uint32_t *dev_items = (uint32_t *)(h + off_items);
        uint32_t *imp = (uint32_t *)(h + off_imp);
        memcpy(h + off_rowslot, row_slot.data(), 4 * (size_t)batch);
        uint32_t en_at = 0, pe_at = 0, so_at = 0, it_at = 0, k_imp = 0;
        for (int r = 0; r < nb; r++) {
            zf_state *st = states[miss_rows[r]];
            const CurrentSet cs = current_set(st);
            StoreRow sr{};
            sr.ent_off = en_at;
            if (use_cache) {
                sr.n_ent = current_set_entries(e->tab, cs.items, cs.n, ents + en_at); sr.flags |= STORE_ROW_CACHE;
                if (sr.n_ent <= (uint32_t)STORE_ROW_ENT) memcpy(sr.ent, ents + en_at, 4 * sr.n_ent);
            }
            row_n_ent[r] = sr.n_ent; row_ent_at[r] = en_at; row_n_items[r] = cs.n;
            en_at += sr.n_ent;
            n_cache_rows += sr.n_ent;
            // the state's name in the host automaton, when it has one there: the key to its name on the device
            const uint32_t named = row_named[r];
            if (!named && host_name_valid(e, st)) rec.host[r] = st->host_id;
            const bool known = named != 0 || st->dev_id == STORE_ROOT_ID || (st->dev_id != 0 && st->dev_epoch == d->store_epoch);
            if (named) {                                   // the device knows this very state: nothing to walk, nothing to bring in
                sr.start = named; sr.n_pending = 0; sr.pend_off = pe_at;
            } else if (known) {
                sr.start = st->dev_id; sr.n_pending = (uint32_t)st->pending.size(); sr.pend_off = pe_at;
                if (sr.n_pending && st->pending_token >= 0 && st->dev_id != 0xFFFFFFFDu) {
                    const uint64_t key = (uint64_t)st->dev_id << 32 | ((uint32_t)st->pending_token + 1u);
                    const uint32_t to = d->hop_find(key);
                    if (to) { sr.start = to; sr.n_pending = 0; }           // somebody has walked this token from this state before
                    else rec.hop[r] = key;
                }
                if (sr.n_pending) memcpy(pend + pe_at, st->pending.data(), sr.n_pending);
                if (sr.n_pending <= (uint32_t)STORE_ROW_PEND) memcpy(sr.pend, st->pending.data(), sr.n_pending);
                pe_at += sr.n_pending;
            } else {
                const Chart &c = chart_of(st);
                const std::vector<uint32_t> &k = packed[miss_rows[r]];
                sr.flags |= STORE_ROW_IMPORTED;
                rows[k_imp] = RowChart{c.n_sets(), so_at, it_at, 0, 0, (uint32_t)c.items.size(), {0, 0}};
                memcpy(so + so_at, k.data() + 1, 4 * c.set_off.size());
                memcpy(dev_items + 2 * (size_t)it_at, k.data() + 1 + c.set_off.size(), 8 * c.items.size());
                so_at += (uint32_t)c.set_off.size(); it_at += (uint32_t)c.items.size();
                imp[k_imp++] = (uint32_t)r;
                st->pending.clear(); st->pending_base = st->fed_total;     // the chart holds everything fed so far
            }
            srow[r] = sr;
            d->h_row_out[(size_t)slot * MAX_BATCH + r] = 0;        // "not reported": the kernel writes the state the row arrives at
            if (use_mini) {
                StoreRowMini &m = mini.r[r];
                bool fits = sr.n_pending <= (uint32_t)STORE_MINI_PEND && sr.n_ent <= (uint32_t)STORE_MINI_ENT;
                for (uint32_t k = 0; fits && k < sr.n_ent; k++) fits = sr.ent[k] < 65536u;
                m.start = sr.start;
                if (fits) {
                    m.meta = sr.n_pending | sr.n_ent << 8 | sr.flags << 16;
                    memcpy(m.pend, sr.pend, STORE_MINI_PEND);
                    for (uint32_t k = 0; k < (uint32_t)STORE_MINI_ENT; k++) m.ent[k] = k < sr.n_ent ? (uint16_t)sr.ent[k] : (uint16_t)0;
                } else m.meta = (sr.flags | STORE_ROW_SPILL) << 16;
                m.spare = 0;
            }
            dst[r] = sc ? row_slot[miss_rows[r]] : miss_rows[r];
            rec.st[r] = st->link; rec.gen[r] = st->generation; rec.upto[r] = st->fed_total;
        }
    }
    MaskArgs a{};
    a.tab = d->tab;
    a.store = d->store;
    const bool direct = !sc;                              // the kernels read the pinned slot in place
    uint8_t *base = direct ? (uint8_t *)d->h_stage[slot] : (uint8_t *)d->d_chart;
    a.store_rows = (const StoreRow *)(base + off_srow);
    a.entries = (const uint32_t *)(base + off_ent);
    a.store_pending = base + off_pend;
    a.store_import_root = d->d_import_root;
    a.store_row_out = d->h_row_out + (size_t)slot * MAX_BATCH;
    a.store_row_dev = d->d_row_out + (size_t)slot * MAX_BATCH;
    a.rows = (const RowChart *)(base + off_rows);
    a.set_off = (const uint32_t *)(base + off_so);
    a.items = (const Item *)(base + off_items);
    a.rank_mask = nullptr;                                // this kernel writes token-order rows itself: no rank-ordered bitmap, no closing kernel
    a.out_mask = sc ? d->d_pool : d_mask;
    a.dst_row = direct ? nullptr : (const uint32_t *)(base + off_dst);
    a.row_slot = (const uint32_t *)(base + off_rowslot);
    a.user_mask = d_mask;
    a.user_batch = batch;
    a.handoff_in_permute = 0;
    a.handoff_in_store = sc ? 0 : 1;                      // with the state cache on, the gather is the call's last kernel
    a.store_mini = use_mini ? 1 : 0;
    if (g_apply.out && direct && nb == batch) {            // every row runs through the kernel, row r of the call is row r of the tensors
        const size_t esz = g_apply.dtype == 0 ? 4 : 2;
        const bool pieces = (uintptr_t)g_apply.logits % 16 == 0 && (uintptr_t)g_apply.out % 16 == 0 && (g_apply.stride * (int64_t)esz) % 16 == 0 &&
                            (size_t)e->V % (16 / esz) == 0;
        if (pieces) {
            a.apply_logits = g_apply.logits; a.apply_out = g_apply.out; a.apply_stride = g_apply.stride; a.apply_dtype = g_apply.dtype;
            g_apply.fused = true;
        }
    }
    a.counters = d->d_counters + COUNTER_SET_WORDS * d->call_parity;
    a.counters_next = d->d_counters + COUNTER_SET_WORDS * (d->call_parity ^ 1u);
    d->call_parity ^= 1u;
    a.host_status = d->h_status + 8 * slot;
    if (++d->call_seq == 0) d->call_seq = 1;
    a.seq = d->call_seq;
    a.fb_waves = FB_WAVES; a.fb_stride = FB_ITEMS_PER_WAVE;   // the closing kernel's fallback pass has nothing to do on this path
    a.batch = nb;
    a.mode = d->mode;
    a.aut_wide = biggest_set > (size_t)AUT_NARROW_SET_MAX ? 1 : 0;   // a hint: which variant of the byte step to try first on larger sets
    {   // LDS of a block: the staged tables, the cache of table entries, and per wavefront the set under construction
        int scratch = e->lane_cap_auto ? (int)std::min<size_t>(LANE_CAP_MAX, (4 * widest + 128 + 31) / 32 * 32) : e->opt.lane_item_cap;
        while (scratch > 32 && store_lds_bytes(d->tab, d->mode, scratch) > (uint32_t)STORE_LDS_MAX) scratch -= 32;
        if (store_lds_bytes(d->tab, d->mode, scratch) > (uint32_t)STORE_LDS_MAX) return fail(ZF_ERR_INVALID_ARG, "the grammar tables leave no LDS for the mask kernel");
        a.aut_scratch = scratch;
        // Blocks per row.  A wavefront takes the row's mask words in segments (16 words = 512 tokens, fewer for rows most of
        // whose tokens are undecided, so that a segment holds about one batch) and the undecided tokens among them 64 at a
        // time; rows differ by orders of magnitude in how many tokens their token-mask cache rows leave undecided, which
        // set-up counted per cache row.  The grid is never larger than what the chip holds at once: a block that had to wait
        // for a place would start from nothing (LDS cache, the row's state) when the others are nearly done, which costs more
        // than a few more passes of the wavefronts that are there.
        const int budget = std::max(nb, std::min(STORE_BLOCKS_PER_CU, store_blocks_per_cu(d->tab, d->mode, scratch)) * std::max(1, d->cus));
        if (!use_mini) {
            const int n_seg = (d->tab.W + STORE_SEG_WORDS - 1) / STORE_SEG_WORDS;
            a.store_uniform_parts = std::max(1, std::min(std::max(1, (n_seg + STORE_WAVES - 1) / STORE_WAVES), budget / nb));
        } else {
            double cost[STORE_MINI_ROWS], inv_cost[STORE_MINI_ROWS];
            int segs[STORE_MINI_ROWS], parts[STORE_MINI_ROWS], seg_w[STORE_MINI_ROWS];
            for (int r = 0; r < nb; r++) {
                double und = d->tab.V;
                if (use_cache && row_n_items[r] <= 64) {
                    const uint32_t n = row_n_ent[r];              // the row's cache-row numbers, as gathered for its record
                    const uint32_t *ent = (const uint32_t *)((uint8_t *)d->h_stage[slot] + off_ent) + row_ent_at[r];
                    uint64_t sig = 0xCBF29CE484222325ull ^ n;
                    for (uint32_t k = 0; k < n; k++) sig = (sig ^ ent[k]) * 0x100000001B3ull;
                    auto it = d->undecided_of.find(sig);
                    if (it == d->undecided_of.end()) {
                        const size_t Wt = (size_t)d->tab.W;
                        uint32_t cnt = 0;
                        for (size_t w = 0; w < Wt; w++) {
                            uint32_t v = 0, cd = 0;
                            for (uint32_t k = 0; k < n; k++) { v |= d->h_valid_tok[ent[k] * Wt + w]; cd |= d->h_cd_tok[ent[k] * Wt + w]; }
                            cnt += (uint32_t)__builtin_popcount(cd & ~v);
                        }
                        if (d->undecided_of.size() > 65536) d->undecided_of.clear();
                        it = d->undecided_of.emplace(sig, cnt).first;
                    }
                    und = it->second;
                }
                // words per segment: as many as are expected to hold 48 undecided tokens, at most 64 (a batch is 64: the
                // tokens are spread unevenly, and a second, nearly empty batch costs as much as a full one)
                const uint32_t seg_words = (uint32_t)std::max(1.0, std::min<double>(STORE_SEG_WORDS_MAX, 48.0 * std::max(1, d->tab.V) / (32.0 * std::max(und, 1.0))));
                segs[r] = (d->tab.W + (int)seg_words - 1) / (int)seg_words;
                seg_w[r] = (int)seg_words;
                // what a pass costs a wavefront (microseconds, measured): an empty segment 2.8, a segment with a batch 3.7, each further batch 3
                const double per_seg = und / segs[r];
                cost[r] = per_seg < 1.0 ? 2.8 + 0.9 * per_seg : 3.7 + 3.0 * std::max(0.0, per_seg / 64.0 - 0.75);
                inv_cost[r] = 1.0 / cost[r];
            }
            // Every wavefront of a row takes the same number of passes (a row is as slow as its slowest wavefront).  The
            // smallest time T is looked for in which every row, taking as many passes as fit into T, leaves the grid within
            // what the chip holds; rows are then given passes back while blocks are left.
            int passes[STORE_MINI_ROWS];
            auto blocks_for = [&](int r, int n_pass) { return std::max(1, (segs[r] + n_pass * STORE_WAVES - 1) / (n_pass * STORE_WAVES)); };
            auto need = [&](double T) {
                int tot = 0;
                for (int r = 0; r < nb; r++) tot += blocks_for(r, std::max(1, (int)(T * inv_cost[r])));
                return tot;
            };
            double lo = cost[0];
            for (int r = 1; r < nb; r++) lo = std::min(lo, cost[r]);
            double hi = lo;
            if (need(hi) > budget) {
                while (need(hi) > budget && hi < 1e9) { lo = hi; hi *= 2; }
                for (int it = 0; it < 6; it++) { const double mid = 0.5 * (lo + hi); if (need(mid) <= budget) hi = mid; else lo = mid; }   // to 2 %: the blocks left over go back to the rows below
            }
            int all = 0;
            for (int r = 0; r < nb; r++) { passes[r] = std::max(1, (int)(hi * inv_cost[r])); parts[r] = blocks_for(r, passes[r]); all += parts[r]; }
            for (int r = 0; r < nb && all < budget; r++) {
                if (passes[r] <= 1) continue;
                const int p = blocks_for(r, passes[r] - 1);
                if (p - parts[r] <= budget - all) { all += p - parts[r]; parts[r] = p; passes[r]--; }
            }
            // Blocks are dealt to the eight XCDs in turn, and every XCD has an L2 of its own.  When rows start at multiples of eight,
            // the blocks that take the same stretch of the vocabulary for different rows run on the same XCD and find each other's
            // strings and cache rows in its L2.  So rows of eight blocks or more are rounded UP to a multiple of eight while blocks are
            // left over (never down: fewer blocks would mean more passes); a block beyond the row's segments leaves at once.
            for (int r = 0; r < nb; r++) {
                const int up = (8 - (parts[r] & 7)) & 7;
                if (parts[r] >= 8 && up && all + up <= budget) { parts[r] += up; all += up; }
            }
#ifndef ZF_MERGE_SEGMENTS
#define ZF_MERGE_SEGMENTS 1
#endif
            for (int r = 0; r < nb; r++) {
                // A wavefront that has several segments to take takes them as fewer, wider ones (up to 64 words): the strings of a
                // segment's first batch are waited for, those of its further batches travel while the batch before is checked.
                if (ZF_MERGE_SEGMENTS && passes[r] > 1 && seg_w[r] < STORE_SEG_WORDS_MAX) {
                    const int words_per_wave = (d->tab.W + parts[r] * STORE_WAVES - 1) / (parts[r] * STORE_WAVES);
                    const int n_pass = (words_per_wave + STORE_SEG_WORDS_MAX - 1) / STORE_SEG_WORDS_MAX;
                    seg_w[r] = std::max(seg_w[r], std::min<int>(STORE_SEG_WORDS_MAX, (words_per_wave + n_pass - 1) / n_pass));
                }
                mini.r[r].meta |= (uint32_t)(seg_w[r] - 1) << 24;
            }
            uint32_t at = 0;
            for (int r = 0; r < nb; r++) { a.store_first_block[r] = (uint16_t)at; at += (uint32_t)parts[r]; }
            for (int r = nb; r < STORE_MINI_ROWS + 8; r++) a.store_first_block[r] = r == nb ? (uint16_t)at : (uint16_t)0xFFFF;   // the kernel compares against all of them
            a.store_uniform_parts = 0;
        }
    }
    const bool prof = d->profiling;
    d->report.chart_bytes = (int64_t)total;
    d->report.cache_rows = (int32_t)n_cache_rows;
    d->report.main_ms = d->report.fallback_ms = d->report.permute_ms = 0.f;
    d->report.overflow_chunks = d->report.walk_chunks = d->report.parser_steps = 0;
    if (!direct) HIP_TRY(launch_upload(d->h_stage[slot], d->d_chart, total, stream));
    if (n_imp) HIP_TRY(launch_store_import(a, (const uint32_t *)(base + off_imp), (uint32_t)n_imp, stream));
    const bool run_kernels = nb > 0;
    if (prof) HIP_TRY(hipEventRecord(d->ev[0], stream));
    d->closing_kernel = sc;
    if (run_kernels) HIP_TRY(launch_mask_store(a, mini, stream));
    if (prof) HIP_TRY(hipEventRecord(d->ev[1], stream));
    if (sc) HIP_TRY(launch_gather(a, stream));
    if (prof) HIP_TRY(hipEventRecord(d->ev[3], stream));
    HIP_TRY(hipEventRecord(d->stage_done[slot], stream));
    d->next_slot = (slot + 1) % DeviceSide::N_SLOTS;
    d->pending++;
    d->last_seq = a.seq; d->last_slot = slot;
    if (!wait) return ZF_OK;
    HIP_TRY(hipStreamSynchronize(stream));
    return zf_mask_wait(e, hip_stream);
}

static void forget_cached_masks(DeviceSide *d) {
    d->cache_index.clear();
    for (auto &ce : d->cache) ce.used = false;
}

// A call that fails part-way may have registered cache slots whose masks were never written.
static int enqueue_mask(zf_engine *e, zf_state *const *states, int32_t batch, uint32_t *d_mask, void *hip_stream, bool wait, bool noalloc = false) {
    DeviceSide *d = e ? e->dev : nullptr;
    bool per_block = false;                               // persistent automaton on hold after a call it had no room for
    if (d && e->store_on && d->store_backoff) { d->store_backoff--; per_block = true; }
    int rc = enqueue_mask_impl(e, states, batch, d_mask, hip_stream, wait, noalloc, per_block);
    if (rc != ZF_OK && d) forget_cached_masks(d);
    if (rc == ZF_ERR_OVERFLOW && d && e->store_on && !noalloc && !per_block) {
        // A set outgrew a wavefront's scratch, or the store filled up within one call.  The waiting call answers through the
        // per-block automaton, whose fallback pass has room in global memory; either way the next calls go that way too,
        // for longer each time it happens, and the store starts over when it is used again.
        d->store_dirty = true;
        d->store_backoff = d->store_backoff_next;
        d->store_backoff_next = std::min<uint32_t>(1024, d->store_backoff_next * 2);
        if (wait) {
            rc = enqueue_mask_impl(e, states, batch, d_mask, hip_stream, wait, noalloc, true);
            if (rc != ZF_OK) forget_cached_masks(d);
        }
    }
    return rc;
}

int zf_compute_mask(zf_engine *e, zf_state *const *states, int32_t batch, uint32_t *d_mask, void *hip_stream) {
    return enqueue_mask(e, states, batch, d_mask, hip_stream, true);
}

// What the persistent automaton holds when a decode loop starts (zf_options.precompute_states).  The automaton is explored
// breadth first from the state of the empty prefix, one byte class at a time (every DFA treats the bytes of a class alike, so one
// byte per class stands for all), on the host and, by computing the mask at every state found, on the device: a mask call
// computes every transition its walk of the vocabulary needs, so the device learns the states a token's length ahead of the
// exploration.  The exploration ends when no new state turns up -- a grammar without recursion has a finite automaton, which is
// then built whole, as engines for regular constraints build theirs when they compile -- or at the budget of states or of
// time, or when the store is a quarter full.  It uses the library's own calls and nothing else (states, advance by bytes, compute_mask): what it leaves behind is
// what a decode loop that happened to visit these prefixes would have left.  Failures are not errors: the engine then starts
// with whatever was learnt, or with nothing, as it did before there was an exploration.
static void explore_from_the_empty_prefix(zf_engine *e) {
    if (!e || !e->store_on || !e->dev || !e->host_aut || e->opt.precompute_states <= 0) return;
    DeviceSide *d = e->dev;
    if (d->pending != 0) return;                          // calls in flight: the store is cleared lazily, and starts empty
    const auto t0 = std::chrono::steady_clock::now();
    auto spent = [&]() { return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count(); };
    const double budget_s = 1.0;
    const size_t budget_states = (size_t)e->opt.precompute_states;
    hipError_t he = hipSetDevice(e->opt.device);
    uint32_t *d_tmp = nullptr;
    constexpr int ROWS = STORE_MINI_ROWS;
    if (he != hipSuccess || hipMalloc((void **)&d_tmp, (size_t)ROWS * (size_t)std::max(e->W, 1) * 4) != hipSuccess) { (void)hipGetLastError(); return; }
    std::vector<uint8_t> rep(std::max(e->tab.n_cls, 0), 0);   // one byte of every class
    std::vector<char> have(rep.size(), 0);
    for (int b = 0; b < 256; b++) { const int c = e->tab.cls[b]; if (c >= 0 && c < (int)rep.size() && !have[c]) { have[c] = 1; rep[c] = (uint8_t)b; } }
    // Breadth first, 64 states at a time: the masks at the states in hand (the device meets them and everything a token's length
    // ahead; the host then knows their names on the device), then the states one byte further, which inherit their parent's
    // name and one pending byte.
    std::vector<zf_state *> queue, edges;
    size_t head = 0;
    std::unordered_set<uint32_t> seen;
    zf_state *root = nullptr;
    bool ok = zf_state_new(e, &root) == ZF_OK;
    if (ok) { queue.push_back(root); seen.insert(HostAutomaton::ROOT); }
    const uint32_t epoch = e->host_epoch;
    while (ok && head < queue.size() && spent() < budget_s) {
        const size_t n = std::min<size_t>(ROWS, queue.size() - head);
        ok = enqueue_mask(e, queue.data() + head, (int32_t)n, d_tmp, nullptr, true) == ZF_OK;
        for (size_t k = head; ok && k < head + n; k++) {
            for (size_t c = 0; c < rep.size() && seen.size() < budget_states; c++) {
                if (!have[c]) continue;
                zf_state *child = nullptr;
                if (zf_state_clone(queue[k], &child) != ZF_OK) { ok = false; break; }
                const bool alive = zf_advance_bytes(child, &rep[c], 1) == ZF_OK && e->host_epoch == epoch &&
                                   child->host_id != HostAutomaton::SINK && child->host_id != HostAutomaton::DEAD;
                if (alive && seen.insert(child->host_id).second) queue.push_back(child);
                else if (alive) edges.push_back(child);   // a way into a state met before: the device has to have walked it too
                else zf_state_destroy(child);
            }
            zf_state_destroy(queue[k]);
            queue[k] = nullptr;
        }
        head += n;
        // the transitions that led to states met before: a row that takes one has the device walk it (its mask is made of look-ups,
        // or is the first visit of a state whose turn in the queue comes later)
        while (ok && edges.size() >= (size_t)ROWS) {
            ok = enqueue_mask(e, edges.data() + edges.size() - ROWS, ROWS, d_tmp, nullptr, true) == ZF_OK;
            for (int k = 0; k < ROWS; k++) { zf_state_destroy(edges.back()); edges.pop_back(); }
        }
        if (e->host_epoch != epoch) ok = false;           // the host automaton filled up and started over: enough
        // a quarter of the store is the most the exploration takes: the store starts over when it is half full, and what a
        // decode loop adds needs room
        if (d->store_states > d->store.cap_states / 4 || d->store_items > d->store.cap_items / 4) break;
    }
    if (ok && !edges.empty() && spent() < budget_s) (void)enqueue_mask(e, edges.data(), (int32_t)edges.size(), d_tmp, nullptr, true);
    for (zf_state *st : edges) zf_state_destroy(st);
    for (zf_state *st : queue) if (st) zf_state_destroy(st);
    (void)hipFree(d_tmp);
    g_err.clear();                                        // a rejected byte is how a dead class shows: not the caller's error
    if (d->store_backoff) {                               // a state the store had no room for: the engine starts as if nothing had been explored
        d->store_backoff = 0; d->store_backoff_next = 8; d->store_dirty = true;
    }
}

int zf_compute_mask_noalloc(zf_engine *e, zf_state *const *states, int32_t batch, uint32_t *d_mask, void *hip_stream) {
    if (e && e->dev && e->dev->pending) return fail(ZF_ERR_INVALID_ARG, "zf_compute_mask_noalloc: asynchronous mask calls are in flight: call zf_mask_wait first");
    return enqueue_mask(e, states, batch, d_mask, hip_stream, true, true);
}

int zf_compute_mask_async(zf_engine *e, zf_state *const *states, int32_t batch, uint32_t *d_mask, void *hip_stream) {
    return enqueue_mask(e, states, batch, d_mask, hip_stream, false);
}

int zf_compute_mask_apply_async(zf_engine *e, zf_state *const *states, int32_t batch, uint32_t *d_mask, const void *d_logits, void *d_out,
                                int32_t dtype, int64_t row_stride, void *hip_stream) {
    if (!e || !d_logits || !d_out || (dtype != 0 && dtype != 1) || row_stride < (e ? e->V : 0)) return fail(ZF_ERR_INVALID_ARG, "bad argument");
    g_apply = ApplyRequest{d_logits, d_out, row_stride, dtype, false};
    const int rc = enqueue_mask(e, states, batch, d_mask, hip_stream, false);
    const bool fused = g_apply.fused;
    g_apply = ApplyRequest{};
    if (rc != ZF_OK || fused) return rc;
    return zf_apply_mask(e, d_logits, d_out, dtype, batch, row_stride, d_mask, hip_stream);   // the other mask kernels, the state cache, odd shapes: two launches
}

int zf_mask_wait(zf_engine *e, void *hip_stream) {
    if (!e || !e->dev) return fail(ZF_ERR_INVALID_ARG, "bad argument");
    DeviceSide *d = e->dev;
    HIP_TRY(hipSetDevice(d->device));
    volatile uint32_t *st = d->h_status;
    if (d->pending) {
        // The newest call's last kernel writes the call's number into pinned memory after its counters: poll that word
        // instead of synchronising the stream (which also waits for whatever the caller queued behind the mask kernels,
        // apply_mask for one, and wakes up microseconds later).  Calls of one engine run in stream order, so the older
        // calls in flight have finished too.  Bounded: after two seconds the stream is synchronised, which also
        // surfaces a device error.
        volatile uint32_t *flag = st + 8 * d->last_slot + 4;
        const auto t0 = std::chrono::steady_clock::now();
        for (uint32_t spins = 0; *flag != d->last_seq; spins++) {
            __builtin_ia32_pause();
            if ((spins & 0xFFFu) == 0xFFFu && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(2)) {
                HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
                if (*flag != d->last_seq) return fail(ZF_ERR_DEVICE, "the mask kernels did not report back");
                break;
            }
        }
        std::atomic_thread_fence(std::memory_order_acquire);
        if (d->profiling) HIP_TRY(hipEventSynchronize(d->ev[3]));
    } else {
        HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));   // nothing of this engine in flight: plain stream synchronisation
    }
    uint32_t unresolved = 0;
    if (e->store_on) {
        // note where every row of the finished calls stands in the persistent automaton, oldest call first
        for (int i = 0; i < DeviceSide::N_SLOTS; i++) {
            const uint32_t k = (d->next_slot + i) % DeviceSide::N_SLOTS;
            DeviceSide::CallRecord &rec = d->rec[k];
            if (!rec.active) continue;
            rec.active = false;
            struct Release { DeviceSide::CallRecord &r; ~Release() { r.st.clear(); } } release{rec};
            const bool good = st[8 * k + 2] == 0 && rec.epoch == d->store_epoch;
            const uint32_t *out = d->h_row_out + (size_t)k * MAX_BATCH;
            for (size_t r = 0; r < rec.st.size() && good; r++) {
                zf_state *s = rec.st[r] ? rec.st[r]->s : nullptr;
                if (out[r] == 0 || (out[r] >= d->store.cap_states && out[r] != 0xFFFFFFFDu)) continue;
                if (rec.hop[r]) d->hop_note(rec.hop[r], out[r]);          // a fact about the automaton, whatever has become of the row
                if (r < rec.host.size() && rec.host[r] && out[r] != 0xFFFFFFFDu) d->name_note(rec.host[r], rec.host_epoch, rec.epoch, out[r]);   // and so is this
                if (!s || s->generation != rec.gen[r]) continue;
                if (rec.upto[r] < s->pending_base) continue;              // a later call's result is already in
                const size_t drop = std::min<size_t>((size_t)(rec.upto[r] - s->pending_base), s->pending.size());
                s->pending_token = -1;
                s->pending.erase(s->pending.begin(), s->pending.begin() + drop);
                s->pending_base = rec.upto[r];
                s->dev_id = out[r]; s->dev_epoch = rec.epoch;
            }
            if (st[8 * k + 5]) { d->store_states = st[8 * k + 5]; d->store_items = st[8 * k + 6]; }
            if (st[8 * k + 7] || st[8 * k + 2]) d->store_dirty = true;    // the store refused a request, or a walk failed: start over
            st[8 * k + 5] = st[8 * k + 6] = st[8 * k + 7] = 0;
        }
    }
    for (int k = 0; k < DeviceSide::N_SLOTS; k++) {
        unresolved += st[8 * k + 2];
        if (st[8 * k + 0] || st[8 * k + 1]) { d->report.overflow_chunks = st[8 * k + 0]; d->report.walk_chunks = st[8 * k + 1]; d->report.parser_steps = st[8 * k + 3]; }
        st[8 * k + 0] = st[8 * k + 1] = st[8 * k + 2] = st[8 * k + 3] = 0;
    }
    if (d->pending && d->profiling) {
        (void)hipEventElapsedTime(&d->report.main_ms, d->ev[0], d->ev[1]);
        d->report.fallback_ms = 0.f;                      // the fallback pass is part of the closing kernel
        if (d->closing_kernel) (void)hipEventElapsedTime(&d->report.permute_ms, d->ev[1], d->ev[3]);
        else d->report.permute_ms = 0.f;                  // the mask kernel was the call's only kernel
    }
    d->pending = 0;
    if (unresolved) forget_cached_masks(d);               // masks written by the failed call must not be served from the cache
    if (unresolved) return fail(ZF_ERR_OVERFLOW, std::to_string(unresolved) + " trie chunks exceeded the fallback arena");
    return ZF_OK;
}

int zf_engine_clear_state_cache(zf_engine *e) {
    if (!e) return fail(ZF_ERR_INVALID_ARG, "null argument");
    if (e->dev) { forget_cached_masks(e->dev); e->dev->store_dirty = true; }   // the persistent automaton starts over as well
    if (e->host_aut) {                                    // and so does the host's: the states find their way back through their charts
        std::unique_lock<std::mutex> lk(e->host_mu);
        while (e->host_walkers != 0) { lk.unlock(); std::this_thread::yield(); lk.lock(); }   // somebody is at work on a transition (and waits for nobody)
        e->host_aut->clear();
        e->host_epoch++;
    }
    explore_from_the_empty_prefix(e);                     // back to what the engine knew when it was compiled
    return ZF_OK;
}

int zf_last_mask_report(const zf_engine *e, zf_mask_report *out) {
    if (!e || !out || !e->dev) return fail(ZF_ERR_INVALID_ARG, "bad argument");
    *out = e->dev->report;
    return ZF_OK;
}

int zf_engine_set_profiling(zf_engine *e, int32_t on) {
    if (!e || !e->dev) return fail(ZF_ERR_INVALID_ARG, "bad argument");
    HIP_TRY(hipSetDevice(e->dev->device));
    if (on) for (auto &ev : e->dev->ev) if (!ev) HIP_TRY(hipEventCreate(&ev));
    e->dev->profiling = on != 0;
    return ZF_OK;
}

int zf_apply_mask(zf_engine *e, const void *d_logits, void *d_out, int32_t dtype, int32_t batch,
                  int64_t row_stride, const uint32_t *d_mask, void *hip_stream) {
    if (!e || !d_logits || !d_out || !d_mask || batch <= 0 || (dtype != 0 && dtype != 1) || row_stride < e->V)
        return fail(ZF_ERR_INVALID_ARG, "bad argument");
    if (!e->dev) return fail(ZF_ERR_DEVICE, "engine was compiled without a device (device = -1)");
    HIP_TRY(hipSetDevice(e->dev->device));
    if (e->V == 0) return ZF_OK;
    HIP_TRY(launch_apply_mask(d_logits, d_out, dtype, batch, row_stride, e->V, e->W, d_mask, (hipStream_t)hip_stream));
    return ZF_OK;
}

}  // extern "C"
