// Interface between the host API code and the HIP kernels.
#pragma once
#include <hip/hip_runtime_api.h>
#include "zf_device.h"

namespace zf {

static const int LANE_CAP_MAX = 24;        // Earley items a lane of the main kernel can hold (LDS)
static const int LANE_DEPTH_MAX = 16;      // trie depth a lane of the main kernel can follow
static const int FB_LANES = 4096;          // lanes of the fallback grid
static const int FB_ITEMS_PER_LANE = 8192; // fallback arena: items per lane (global memory)
static const int FB_DEPTH_MAX = 256;

struct MaskArgs {
    DeviceTables tab;
    const RowChart *rows;      // [batch]
    const uint32_t *set_off;   // shared CSR offsets of all rows' sets
    const Item *items;         // shared item array of all rows
    uint32_t *rank_mask;       // [batch][Wr] verdicts in trie (rank) order
    uint32_t *out_mask;        // [batch][W] verdicts in token-id order
    uint32_t *counters;        // [0] overflow entries, [1] entries the fallback could not resolve
    uint2 *overflow_list;      // (row, chunk)
    uint32_t overflow_cap;
    uint2 *fb_items;           // [FB_ITEMS_PER_LANE][FB_LANES] interleaved
    uint32_t *fb_set_start;    // [FB_DEPTH_MAX + 2][FB_LANES]
    int32_t batch;
    int32_t lane_cap;
};

hipError_t launch_mask_main(const MaskArgs &a, hipStream_t s);
hipError_t launch_mask_fallback(const MaskArgs &a, hipStream_t s);
hipError_t launch_permute(const MaskArgs &a, hipStream_t s);
hipError_t launch_apply_mask(const void *logits, void *out, int dtype, int batch, int64_t row_stride, int V, int W,
                             const uint32_t *mask, hipStream_t s);

}  // namespace zf
