// Interface between the host API code and the HIP kernels.
#pragma once
#include <hip/hip_runtime_api.h>
#include "zf_device.h"

namespace zf {

static const int LANE_CAP_MAX = 2048;      // upper limit of the walk kernel's item budget per wavefront (LDS)
static const int LANE_CAP_DEFAULT = 96; 
static const int WALK_WAVES = 8;           // wavefronts (= queued chunks) per block of the walk kernel; they share the staged tables
static const int WALK_BLOCK = WALK_WAVES * 64;
static const int WALK_RUN_MAX = 2;         // consecutive queue items a wavefront takes at a time (one when the queue is short)
static const int WALK_NODES_LDS = 80;      // trie nodes of a chunk the walk kernel stages in LDS (bigger chunks go to the fallback)
static const int WALK_DEPTH_MAX = 32;      // trie depth the walk kernel follows (deeper paths go to the fallback)
static const int BASE_SETS_LDS = 31;       // a row's chart is staged into LDS when it has at most this many sets ...
static const int BASE_ITEMS_LDS = 64;      // ... and items (the mask-automaton kernel takes larger limits from the host when LDS allows)
static const int AUT_NARROW_SET_MAX = 8;    // charts whose sets are all this small run the kernel build without the wide variant of the byte step
static const int AUT_BASE_SETS_MAX = 1023; // the largest limits the host asks for
static const int AUT_BASE_ITEMS_MAX = 4096;
static const int TABLE_LDS_BUDGET = 56 * 1024;
static const int AUT_WAVES = 8;            // wavefronts per block of the mask-automaton kernel
static const int AUT_BLOCK = AUT_WAVES * 64;
static const int AUT_SUB_WORDS = 128;      // words of the rank-ordered bitmap (32 strings each) a block merges and checks per pass ...
static const int AUT_GROUP_WORDS = 4;      // ... taken from the row in groups of this many neighbouring words (two batches of 64 ranks), dealt to the blocks round robin
static const int AUT_ENT_LDS = 64;         // token-mask-cache rows of the row's current set kept in LDS (more are read from global memory)
static_assert(AUT_NARROW_SET_MAX <= AUT_ENT_LDS, "the kernel build for small sets keeps all cache-row numbers of a row in LDS");
static const int AUT_TABLE_LOADS = (TABLE_LDS_BUDGET + AUT_BLOCK * 16 - 1) / (AUT_BLOCK * 16);   // 16-byte pieces of the staged tables per thread
static const int AUT_HELP_QUEUE = 512;     // transitions one block can leave for free wavefronts in the course of a launch
static const int AUT_STATES_DEFAULT = 64;  // automaton states a block can hold (more when LDS allows and the grammar is small)
static const int AUT_SPIN_LIMIT = 1 << 16; // polls of a transition another wavefront is computing before giving the strings to the fallback
static const int FB_DEPTH_MAX = 256;
static const int FB_WAVES = 512;           // wavefronts of the closing kernel that run the fallback pass (each has its own arena)
static const int FB_ITEMS_PER_WAVE = 65536; // its arena in global memory: items per wavefront (256 MB in all)
// The entry point that may not allocate keeps every per-call device buffer in one static device array:
static const size_t NOALLOC_SCRATCH_BYTES = 16u << 20;
static const int NOALLOC_FB_WAVES = 32;          // its fallback pass: fewer wavefronts ...
static const int NOALLOC_FB_ITEMS_PER_WAVE = 16384;   // ... with smaller arenas (4 MB of the array)
static const size_t NOALLOC_STAGE_BYTES = 256u << 10;  // pinned staging room per slot that every engine has from the start

// The persistent automaton (zf_options.walk_mode = 2): one store per engine in device memory.
#ifndef ZF_STORE_WAVES
#define ZF_STORE_WAVES 4
#endif
#ifndef ZF_STORE_SUB_WORDS
#define ZF_STORE_SUB_WORDS 64
#endif
#ifndef ZF_STORE_LC_BITS
#define ZF_STORE_LC_BITS 10
#endif
static const int STORE_WAVES = ZF_STORE_WAVES;  // wavefronts per block of the mask kernel over the persistent automaton
static const int STORE_BLOCK = STORE_WAVES * 64;
static const int STORE_SUB_WORDS = ZF_STORE_SUB_WORDS;   // words of the rank-ordered bitmap a block merges and checks per pass (at most 128: one wavefront lists the word pairs)
static const int STORE_LDS_MAX = 159 * 1024;   // dynamic LDS a block of that kernel may ask for (the hand-over of the call's status has a static word of its own)
static const int STORE_SEG_WORDS = 16;         // mask words (of 32 tokens) a wavefront merges and checks per pass in calls of more than STORE_MINI_ROWS rows ...
static const int STORE_SEG_WORDS_MAX = 64;     // ... smaller calls choose 1 to 64 per row, so that a pass holds about one batch of undecided tokens
static const int STORE_WARM_ROWS = 32;         // rows of the transition table (states one byte from a row's current state) a block reads ahead into its LDS cache
static const int STORE_LC_BITS = ZF_STORE_LC_BITS;       // log2 of the entries of a block's LDS cache of table entries (8 bytes each)
#ifndef ZF_STORE_BLOCKS_PER_CU
#define ZF_STORE_BLOCKS_PER_CU 3
#endif
static const int STORE_BLOCKS_PER_CU = ZF_STORE_BLOCKS_PER_CU;   // blocks per compute unit the grid is made of at most (fewer when a compute unit holds fewer at once)
static const int STORE_PENDING_LDS = 256;       // pending bytes of a row a block keeps in LDS (more are read from the upload)
static const int STORE_PENDING_MAX = 4096;      // beyond this many bytes since its state was last known a row comes in through its chart again
static const uint32_t STORE_ROW_CACHE = 1u;     // StoreRow::flags: the token-mask cache rows of the row are listed
static const uint32_t STORE_ROW_IMPORTED = 2u;  // the row's start state is the one the import kernel made from its chart
struct StoreView {
    uint2 *hdr;                 // [cap_states] (first item in the arena, item count); count 0xFFFFFFFF = not published
    uint2 *arena;               // [cap_items] (item word, name of the set the item's rule started in)
    uint32_t *trans;            // [cap_states][n_cls] next state or AT_*
    unsigned long long *intern; // [intern_mask + 1] content signature << 32 | state; 0 = free
    uint32_t *ctl;              // [0] states handed out (the next name), [1] items handed out, [2] requests the store had no room for
    uint32_t cap_states, cap_items, intern_mask;
};
static const int STORE_ROW_ENT = 10, STORE_ROW_ENT_AT = 6;      // token-mask-cache rows a record holds inline, and the word they start at
static const int STORE_ROW_PEND = 64, STORE_ROW_PEND_AT = 16;   // pending bytes a record holds inline, and the word they start at
struct StoreRow {               // one row of a call: 128 bytes, read by a wavefront with one load (lane k = word k)
    uint32_t start;             // [0] the state the row was last known to be in
    uint32_t n_pending;         // [1] bytes (as byte classes) fed to the row since then: inline when they fit ...
    uint32_t pend_off;          // [2] ... else at this offset of the call's pending bytes
    uint32_t n_ent, ent_off;    // [3] [4] token-mask-cache rows of the row's current set: inline when they fit, else in MaskArgs::entries
    uint32_t flags;             // [5]
    uint32_t ent[STORE_ROW_ENT];
    uint8_t pend[STORE_ROW_PEND];
};
static_assert(sizeof(StoreRow) == 128, "a wavefront reads a row's record as 32 words");
// The same record in 48 bytes, for calls of up to STORE_MINI_ROWS rows: it travels in the kernel's argument block, which the
// wavefronts read without a trip to the host's memory.  A row whose record does not fit (more pending bytes, more or larger
// cache row numbers) says so in its flags and is read from store_rows.
static const int STORE_MINI_ROWS = 64, STORE_MINI_PEND = 16, STORE_MINI_ENT = 10;
static const uint32_t STORE_ROW_SPILL = 4u;     // flags of a short record: the row's full record is in MaskArgs::store_rows
struct StoreRowMini {
    uint32_t start;                               // as StoreRow::start
    uint32_t meta;                                // n_pending | n_ent << 8 | flags << 16 | (mask words per pass - 1) << 24
    uint8_t pend[STORE_MINI_PEND];
    uint16_t ent[STORE_MINI_ENT];
    uint32_t spare;
};
static_assert(sizeof(StoreRowMini) == 48, "short row records are twelve words");
struct StoreMiniRows { StoreRowMini r[STORE_MINI_ROWS]; };

// A set of per-call counters: words 0-7 as listed at MaskArgs::counters, then the tickets the blocks of a call's last kernel
// draw when they are done (one word per group of blocks, so that thousands of blocks do not queue up at one address, and a
// top word the last block of each group draws from).
// A ticket word is 64 bits: tickets drawn in the low half, and in the high half a partial sum of counter [1] (undecided tokens)
// that the mask kernel over the persistent automaton adds with the same operation, once per block.  (Thousands of additions to
// one word, or to one cache line, queue up at the memory channel that holds it and hold up every other request to that channel:
// 30 us per launch when every wavefront added its count to counters[1].)  The block that hands the status over adds them up.
static const int COUNTER_SET_WORDS = 160, TICKET_GROUPS = 64, TICKET_AT = 16, TICKET_TOP = 144;

struct MaskArgs {
    DeviceTables tab;
    StoreView store;
    const StoreRow *store_rows;        // [batch]
    const uint8_t *store_pending;
    uint32_t *store_import_root;       // [batch] device memory: written by the import kernel
    uint32_t *store_row_out;           // [batch] pinned host memory: the state every row is in after this call's walk ...
    uint32_t *store_row_dev;           // [batch] ... which the mask kernel notes here (device memory); the block that hands the call's status over copies it out
    // The grid of the store kernel is one-dimensional.  In calls of up to STORE_MINI_ROWS rows the host gives rows whose
    // token-mask cache leaves more tokens undecided more blocks: row r has blocks store_first_block[r] .. store_first_block[r + 1]
    // (ascending; 0xFFFF beyond the call's rows) and store_uniform_parts is 0; larger calls give every row store_uniform_parts blocks.
    alignas(16) uint16_t store_first_block[STORE_MINI_ROWS + 8];
    int32_t store_uniform_parts;
    const RowChart *rows;      // [batch]
    const uint32_t *set_off;   // shared CSR offsets of all rows' sets
    const Item *items;         // shared item array of all rows
    const uint32_t *entries;   // shared array of token-mask-cache rows (see RowChart)
    uint32_t so_stride, it_stride, ent_stride;   // not 0: row r's sections start at r * stride in set_off / items / entries (every row has the same room)
    uint32_t *rank_mask;       // [batch][Wr] verdicts in trie (rank) order
    uint32_t *out_mask;        // token-order rows: the caller's tensor, or the state cache's pool
    const uint32_t *dst_row;   // [batch] row of out_mask that row r of this launch is written to; null = row r
    const uint32_t *row_slot;  // [user_batch] pool slot that holds the finished mask of each of the caller's rows
    uint32_t *user_mask;       // the caller's [user_batch][W] tensor (target of the gather)
    int32_t user_batch;
    int32_t handoff_in_permute; // 1: permute is the call's last kernel (state cache off), else the gather is
    int32_t handoff_in_store;  // 1: the mask kernel over the persistent automaton is the call's last kernel (it writes the caller's rows itself)
    // zf_compute_mask_apply_async on that path: a wavefront masks the logits of the tokens whose mask words it has just written
    // (no second kernel); null = the mask only.  Row r of the call is row r of the tensors; 16-byte pieces (V, the row stride
    // and the pointers are multiples of a piece: the host checks).
    const void *apply_logits;
    void *apply_out;
    int64_t apply_stride;      // elements between rows
    int32_t apply_dtype;       // 0 = fp32, 1 = bf16
    int32_t store_mini;        // 1: the rows' records are in the kernel's StoreMiniRows argument
    uint32_t *counters;        // [0] chunks passed to the fallback, [1] length of the work queue, [2] chunks nobody could resolve,
                               // [3] Earley byte steps, [4] fallback wavefronts that have finished, [16..144] tickets of the call's last kernel;
                               // COUNTER_SET_WORDS words per set
    uint32_t *host_status;     // pinned host memory, 8 words: this call's counters [0..3], written by its last kernel, then [4] = seq
    uint32_t seq;              // the call's number (never 0): the last word the call's last kernel writes, which is what the host waits for
    uint32_t *counters_next;   // the next call's counters: cleared by this call's last kernel (no separate memset)
    uint4 *work;               // queue of (row, chunk, undecided strings, -) that need the parser walk
    uint4 *overflow_list;      // (row, chunk, undecided strings, -) for the fallback
    uint32_t overflow_cap;
    uint2 *fb_items;           // [fb_waves][fb_stride]
    uint32_t *fb_set_start;    // [fb_waves][FB_DEPTH_MAX + 2]
    uint32_t fb_waves;         // wavefronts of the fallback pass (each has its own arena) ...
    uint32_t fb_stride;        // ... of this many items
    int32_t batch;
    int32_t lane_cap;          // item budget of a walking wavefront
    int32_t fb_cap;            // item budget of a fallback wavefront (<= FB_ITEMS_PER_WAVE)
    int32_t walk_blocks;       // blocks of the walk grid (one and a half times what the chip holds at once)
    int32_t mode;              // 0: all tables staged in LDS, 1: the small ones only, 2: none
    // mask-automaton kernel: capacities of one block's automaton in LDS
    int32_t aut_states;        // states (rows of the transition table)
    int32_t aut_arena;         // items of all states together
    int32_t aut_scratch;       // items of one set under construction (per wavefront)
    int32_t aut_parts;         // blocks per row (grid.x)
    int32_t aut_base_sets;     // a row's chart is staged into LDS when it has at most this many sets ...
    int32_t aut_base_items;    // ... and items (both at least BASE_SETS_LDS / BASE_ITEMS_LDS)
    int32_t aut_wide;          // 1: some set of some row's chart has more than AUT_NARROW_SET_MAX items (the kernel build with the wide byte step)
};

int choose_table_mode(const DeviceTables &t);
uint32_t walk_lds_bytes(const DeviceTables &t, int mode, int lane_cap);   // dynamic LDS of one block of the walk kernel
hipError_t walk_blocks_per_cu(int mode, uint32_t lds_bytes, int *out);   // resident blocks of the walk kernel per compute unit
hipError_t prepare_kernels();   // one-time function attributes (dynamic LDS above 64 KB) of all kernels:
hipError_t prepare_walk_kernels();
hipError_t prepare_automaton_kernels();
hipError_t launch_upload(const void *pinned_src, void *dst, size_t bytes, hipStream_t s);   // bytes rounded up to 16: both buffers must hold that much
hipError_t launch_cache_merge(const MaskArgs &a, hipStream_t s);
hipError_t launch_mask_walk(const MaskArgs &a, hipStream_t s);
uint32_t automaton_lds_bytes(const DeviceTables &t, int mode, int states, int arena, int scratch, int base_sets, int base_items, bool wide);
hipError_t launch_mask_automaton(const MaskArgs &a, hipStream_t s);
hipError_t prepare_store_kernels();
uint32_t store_lds_bytes(const DeviceTables &t, int mode, int scratch);
int store_blocks_per_cu(const DeviceTables &t, int mode, int scratch);
hipError_t launch_mask_store(const MaskArgs &a, const StoreMiniRows &mini, hipStream_t s);
hipError_t launch_store_clear(const StoreView &G, uint32_t ncls, const void *root_items, uint32_t n_root, hipStream_t s);
hipError_t launch_store_import(const MaskArgs &a, const uint32_t *import_rows, uint32_t n_import, hipStream_t s);
hipError_t launch_finish(const MaskArgs &a, int cus, hipStream_t s);   // fallback pass (when anything was listed) + permutation into token order
hipError_t launch_gather(const MaskArgs &a, hipStream_t s);
// Per-device address of the static device array behind the entry point that may not allocate.
hipError_t scratch_init(int device);            // resolves it once per device; `device` must be current
void *scratch_ptr(int device);                  // null before scratch_init(device) has succeeded
hipError_t launch_clear_words(uint32_t *p, uint32_t n_words, hipStream_t s);   // a fill kernel (no memset node in a captured graph)
hipError_t launch_apply_mask(const void *logits, void *out, int dtype, int batch, int64_t row_stride, int V, int W,
                             const uint32_t *mask, hipStream_t s);

}  // namespace zf
