// Host build of the connection-ordering routine (spdnn_order.h), so that the
// set-up logic can be tested without a GPU.  Not used by the inference path.
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

}  // extern "C"
