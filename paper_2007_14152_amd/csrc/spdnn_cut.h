// How a general layer (neurons of any number of connections, Section II-A-1; the zero padding of Section
// III-A-3 at the granularity of a lane) is cut into workgroups.  Plain C++ for the host: the set-up calls it
// once per layer with the row pointers it has read back, and the host tests call it without a GPU.
//
// A neuron of K connections takes ceil(K / 32) lanes ("parts"); a workgroup takes a run of neighbouring neurons,
// a multiple of 4 (four neighbouring neurons share a 16-byte output store), at most 1024 neurons and at most
// 1024 lanes.  Two cuts:
//  * packed: as many neurons as fill the 1024 lanes, fewer where the next four neurons would widen the
//    workgroup's column window beyond one LDS stage that it still fits;
//  * plain: runs of Gl workgroups (the workgroups that share an XCD at inference: they read the same rows through
//    one window) over Gl * 1024 / P neurons each, P = lanes of the layer's longest neuron rounded up to a power of
//    two; inside a run the workgroups get equally many lanes, not equally many neurons, so that they take equally
//    long and stay within reach of each other in the L2.  A run that cannot be cut that way (a workgroup would
//    overflow) is cut into equal numbers of neurons, which always fits.  Runs are padded with empty workgroups
//    {N, 0} to their full number, so run r always starts at workgroup r * Gl.
// The packed cut is kept if it fits the room there is (P * nblk workgroups) and needs at most three quarters of
// the plain cut's workgroups: its workgroups are fuller, and have no idle waves left for the finishing.
#pragma once
#include <stdint.h>

#include <algorithm>
#include <vector>

namespace spdnn {

struct NeuronRange {
    int first, count;  // {N, 0}: a workgroup without neurons
};

// hp: N + 1 row pointers; qw: for every four neurons {lowest column, highest column} (2 ints each); P: the layer's
// passes; nblk = ceil(N / 1024); G: workgroups of a fixed-32 layer that share an XCD.  N is a multiple of 4.
inline std::vector<NeuronRange> cut_workgroups(const int32_t* hp, const int* qw, int N, int P, int nblk, int G,
                                               int wg_lanes = 1024, int part = 32, int stage_cols = 4096) {
    auto lanes4 = [&](int j) {  // lanes of the four neurons j .. j+3
        int q = 0;
        for (int i = 0; i < 4; ++i) q += (hp[j + i + 1] - hp[j + i] + part - 1) / part;
        return q;
    };
    std::vector<NeuronRange> out;
    {
        int first = 0, lanes = 0, lo = N, hi = -1;
        for (int j = 0; j < N; j += 4) {
            const int q = lanes4(j);
            const int wx = qw[2 * (j / 4)], wy = qw[2 * (j / 4) + 1];
            const int nlo = std::min(lo, wx), nhi = std::max(hi, wy);
            // a workgroup whose columns fit one LDS stage is not widened beyond it
            const bool widens = hi >= lo && hi - (lo & ~3) < stage_cols && nhi - (nlo & ~3) >= stage_cols;
            if (lanes + q > wg_lanes || j - first == wg_lanes || (j > first && widens)) {
                out.push_back(NeuronRange{first, j - first});
                first = j;
                lanes = 0;
                lo = N;
                hi = -1;
            }
            lanes += q;  // a neuron has at most P <= 256 parts: four of them always fit
            lo = std::min(lo, wx);
            hi = std::max(hi, wy);
        }
        out.push_back(NeuronRange{first, N - first});
    }
    // (measured: 128 plain against 112 packed workgroups 13.2 against 15.1 ms per layer, 256 against 144: 27.3
    // against 22.6)
    const int R = wg_lanes / P;
    const size_t plain = (size_t)(N + R - 1) / R;
    if (out.size() <= (size_t)P * nblk && 4 * out.size() <= 3 * plain) return out;

    out.clear();
    int Gl = 1;
    for (int g : {32, 16, 8, 4, 3, 2, 1})
        if (g <= G * P && nblk % g == 0) {
            Gl = g;
            break;
        }
    for (int r0 = 0; r0 < N; r0 += Gl * R) {
        const int r1 = std::min(N, r0 + Gl * R);
        const int nW = (r1 - r0 + R - 1) / R;
        long left = 0;
        for (int j = r0; j < r1; j += 4) left += lanes4(j);
        const size_t mark = out.size();
        int first = r0, lanes = 0, wleft = nW;
        long target = (left + wleft - 1) / wleft;
        for (int j = r0; j < r1; j += 4) {
            const int q = lanes4(j);
            const bool full = lanes + q > wg_lanes || j - first == wg_lanes;
            if (j > first && (full || (wleft > 1 && lanes + q - target > target - lanes))) {
                out.push_back(NeuronRange{first, j - first});
                left -= lanes;
                wleft = std::max(1, wleft - 1);
                target = (left + wleft - 1) / wleft;
                first = j;
                lanes = 0;
            }
            lanes += q;
        }
        out.push_back(NeuronRange{first, r1 - first});
        if (out.size() - mark > (size_t)nW) {  // a workgroup overflowed on the way: the cut by neurons always fits
            out.resize(mark);
            for (int j = r0; j < r1; j += R) out.push_back(NeuronRange{j, std::min(R, r1 - j)});
        }
        while (out.size() - mark < (size_t)nW) out.push_back(NeuronRange{N, 0});
    }
    return out;
}

}  // namespace spdnn
