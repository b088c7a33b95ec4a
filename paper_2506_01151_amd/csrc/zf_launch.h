// Interface between the host API code and the HIP kernels.
#pragma once
#include <hip/hip_runtime_api.h>
#include "zf_device.h"

namespace zf {

static const int LANE_CAP_MAX = 96;        // upper limit of the per-lane item budget (LDS is sized by the budget in use)
static const int LANE_CAP_DEFAULT = 48;
static const int LANE_DEPTH_MAX = 16;      // trie depth a lane of the main kernel can follow
static const int MAIN_BLOCK = 256;         // threads per block of the main kernel (4 wavefronts share the staged tables)
static const int BASE_SETS_LDS = 63;       // a row's chart is staged into LDS when it has at most this many sets ...
static const int BASE_ITEMS_LDS = 192;     // ... and items
static const int TABLE_LDS_BUDGET = 56 * 1024;
static const int FB2_CAP = 2048;           // items of the second-level fallback (one lane per wavefront, list in LDS)
static const int FB2_BLOCKS = 2048;
static const int FB_DEPTH_MAX = 256;
static const int FB3_LANES = 2048;         // lanes of the last-level fallback grid
static const int FB3_ITEMS_PER_LANE = 16384; // its arena in global memory: items per lane

struct MaskArgs {
    DeviceTables tab;
    const RowChart *rows;      // [batch]
    const uint32_t *set_off;   // shared CSR offsets of all rows' sets
    const Item *items;         // shared item array of all rows
    const uint32_t *entries;   // shared array of token-mask-cache rows (see RowChart)
    uint32_t *rank_mask;       // [batch][Wr] verdicts in trie (rank) order
    uint32_t *out_mask;        // [batch][W] verdicts in token-id order
    uint32_t *counters;        // [0] chunks passed to level 2, [1] chunks passed to level 3, [2] unresolved
    uint32_t *row_count;       // [batch] length of each row's queue of chunks that need the parser walk
    uint2 *work;               // [batch][n_chunks] (chunk, undecided strings) queue per row
    uint4 *overflow_list;      // (row, chunk, undecided strings, -) for level 2
    uint4 *overflow_list2;     // same for level 3
    uint32_t overflow_cap;
    uint2 *fb_items;           // [FB3_ITEMS_PER_LANE][FB3_LANES] interleaved
    uint32_t *fb_set_start;    // [FB_DEPTH_MAX + 2][FB3_LANES]
    int32_t batch;
    int32_t lane_cap;
    int32_t fb2_cap;           // item budget of fallback level 2 (<= FB2_CAP)
    int32_t mode;              // 0: all tables staged in LDS, 1: the small ones only, 2: none
};

int choose_table_mode(const DeviceTables &t);
hipError_t prepare_kernels();   // one-time function attributes (dynamic LDS above 64 KB)
hipError_t launch_cache_merge(const MaskArgs &a, hipStream_t s);
hipError_t launch_mask_main(const MaskArgs &a, hipStream_t s);
hipError_t launch_mask_fallback2(const MaskArgs &a, hipStream_t s);
hipError_t launch_mask_fallback3(const MaskArgs &a, hipStream_t s);
hipError_t launch_permute(const MaskArgs &a, hipStream_t s);
hipError_t launch_apply_mask(const void *logits, void *out, int dtype, int batch, int64_t row_stride, int V, int W,
                             const uint32_t *mask, hipStream_t s);

}  // namespace zf
