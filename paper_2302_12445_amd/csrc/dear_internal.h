// Internal definitions shared by the host planner and the HIP side of libdear.
#pragma once

#include <cstdint>
#include <vector>

#include "dear.h"

struct dear_plan_s {
    int32_t L = 0, B = 0, P = 0, g = 0;
    int64_t threshold_bytes = 0;
    int64_t N = 0;               // sum of layer sizes
    int64_t row_len = 0;         // sum of S_b: one worker's row of a shard buffer
    std::vector<int64_t> layer_sizes, layer_offset;
    std::vector<int32_t> layer_bucket;
    std::vector<int32_t> bucket_first_layer, bucket_n_layers;
    std::vector<int64_t> bucket_len, bucket_shard_len, bucket_shard_base;
};

typedef dear_tile_t dear_tile;
static_assert(sizeof(dear_tile) == 32, "tile descriptors are read as two 16-byte loads");

constexpr int DEAR_BLOCK = 256;  // threads per workgroup = 4 wavefronts

// Cuts every bucket of the plan into tiles (plan.cpp).
int64_t dear_emit_tiles(const dear_plan_s &pl, int32_t b_first, int32_t b_last, dear_tile *out,
                        int64_t capacity, int64_t *tile_begin);
void dear_build_tiles(const dear_plan_s &pl, std::vector<dear_tile> &tiles, std::vector<int64_t> &tile_begin);
