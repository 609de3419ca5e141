// Host build of the connection-ordering routine (spdnn_order.h) and of the tile
// layout functions (spdnn_layout.h), so that the set-up logic can be tested without a
// GPU.  Not used by the inference path.
#include "spdnn_cut.h"
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

// pairs: [32][32] bank pair (0..31) of every connection of 32 neighbouring neurons.
// step_of: [32][32] out, step at which connection k of lane l is placed.
// Returns the cost (sum over the 32 steps of the largest pair multiplicity), -1 if a lane got two
// connections in one step or a connection was never placed.
int spdnn_order_group32_host(const uint8_t* pairs, uint8_t* step_of) {
    static spdnn::Order32Scratch S;
    uint8_t at[32][32];  // pair used by lane l at step s
    for (int i = 0; i < 32 * 32; ++i) {
        step_of[i] = 255;
        (&at[0][0])[i] = 255;
    }
    bool bad = false;
    spdnn::order_group32(
        S, [&](int l, int k) -> unsigned { return pairs[l * 32 + k]; },
        [&](int l, int step, int k) {
            if (k < 0 || k > 31 || step_of[l * 32 + k] != 255 || at[l][step] != 255) {
                bad = true;
                return;
            }
            step_of[l * 32 + k] = (uint8_t)step;
            at[l][step] = pairs[l * 32 + k];
        });
    if (bad) return -1;
    int total = 0;
    for (int step = 0; step < 32; ++step) {
        int m[32] = {0}, mx = 0;
        for (int l = 0; l < 32; ++l) {
            if (at[l][step] == 255) return -1;
            if (++m[at[l][step]] > mx) mx = m[at[l][step]];
        }
        total += mx;
    }
    return total;
}

// Tile layout functions, one call per value.
uint32_t spdnn_tile_offset_host(uint32_t slot) { return spdnn::tile_offset(slot); }
uint32_t spdnn_tile_pair_bytes_host(uint32_t cols) { return spdnn::tile_pair_bytes(cols); }
int spdnn_lane_of_group_host(int set, int rank) { return spdnn::lane_of_group(set, rank); }
uint32_t spdnn_set_of_lane_host(uint32_t lane) { return spdnn::set_of_lane(lane); }
uint32_t spdnn_rank_in_set_host(uint32_t lane) { return spdnn::rank_in_set(lane); }
uint32_t spdnn_col_slot_host(uint32_t c) { return spdnn::col_slot(c); }
uint32_t spdnn_store_group_host(uint32_t c) { return spdnn::store_group(c); }
uint32_t spdnn_row2_pos_host(uint32_t c) { return spdnn::row2_pos(c); }
int spdnn_unit_neuron_host(int u, int p, int seg_log2, int seg_stride) { return spdnn::unit_neuron(u, p, seg_log2, seg_stride); }
void spdnn_win_union_host(int ax, int ay, int cx, int cy, int N, int* out) { spdnn::win_union(ax, ay, cx, cy, N, out[0], out[1]); }
int spdnn_win_rel_host(int c, int c_lo, int N) { return spdnn::win_rel(c, c_lo, N); }
int spdnn_win_col_host(int c_lo, int rel, int N) { return spdnn::win_col(c_lo, rel, N); }

// Workgroup cut of a general layer (spdnn_cut.h).  ptr: N + 1 row pointers; qw: 2 * (N / 4) ints, lowest and
// highest column of every four neurons; out: room for cap pairs {first neuron, number of neurons}.  Returns the
// number of workgroups, or -1 if there are more than cap.
int spdnn_cut_workgroups_host(const int32_t* ptr, const int32_t* qw, int N, int P, int nblk, int G, int32_t* out, int cap) {
    const std::vector<spdnn::NeuronRange> cut = spdnn::cut_workgroups(ptr, qw, N, P, nblk, G);
    if ((int)cut.size() > cap) return -1;
    for (size_t i = 0; i < cut.size(); ++i) {
        out[2 * i] = cut[i].first;
        out[2 * i + 1] = cut[i].count;
    }
    return (int)cut.size();
}

}  // extern "C"
