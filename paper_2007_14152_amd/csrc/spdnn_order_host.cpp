// Host build of the connection-ordering routine (spdnn_order.h) and of the tile
// layout functions (spdnn_layout.h), so that the set-up logic can be tested without a
// GPU.  Not used by the inference path.
#include "spdnn_layout.h"
#include "spdnn_order.h"

extern "C" {

// quads: [16][32] quad (0..15) of every connection of 16 neighbouring neurons, 255 = absent.
// step_of: [16][32] out, step at which connection k of lane l is placed (255 if absent).
// nsteps: number of steps (>= the largest number of connections of any lane).
// Returns the cost (sum over steps of the largest quad multiplicity).
int spdnn_order_group_host(const uint8_t* quads, uint8_t* step_of, int nsteps) {
    spdnn::OrderScratch S;
    uint8_t placed[16][32];
    for (int i = 0; i < 16 * 32; ++i) {
        step_of[i] = 255;
        (&placed[0][0])[i] = 255;
    }
    spdnn::order_group(
        S, nsteps, [&](int l, int k) -> unsigned { return quads[l * 32 + k]; },
        [&](int l, int step, int k) {
            step_of[l * 32 + k] = (uint8_t)step;
            placed[l][step] = quads[l * 32 + k];
        });
    return spdnn::order_cost([&](int l, int step) -> unsigned { return placed[l][step]; });
}

// Cost of the order as given (connection k at step k).
int spdnn_order_cost_host(const uint8_t* quads) {
    return spdnn::order_cost([&](int l, int step) -> unsigned { return quads[l * 32 + step]; });
}

// Tile layout functions, one call per value.
uint32_t spdnn_tile_offset_host(uint32_t slot) { return spdnn::tile_offset(slot); }
uint32_t spdnn_tile_pair_bytes_host(uint32_t cols) { return spdnn::tile_pair_bytes(cols); }
int spdnn_lane_of_group_host(int set, int rank) { return spdnn::lane_of_group(set, rank); }
uint32_t spdnn_set_of_lane_host(uint32_t lane) { return spdnn::set_of_lane(lane); }
uint32_t spdnn_rank_in_set_host(uint32_t lane) { return spdnn::rank_in_set(lane); }
uint32_t spdnn_col_slot_host(uint32_t c) { return spdnn::col_slot(c); }
uint32_t spdnn_store_group_host(uint32_t c) { return spdnn::store_group(c); }

}  // extern "C"
