// Bank-aware ordering of each output neuron's 32 connections (part of the weight
// set-up, a0).  Plain C++ usable on the host and in device code.
//
// Why.  In the fused kernel lane = output neuron and step k of a tile makes every
// lane read the 16-byte LDS entry of its k-th connection's column.  gfx950 serves
// 16 lanes of a ds_read_b128 per clock from 64 four-byte banks, i.e. from 16
// "quads" of 16 bytes; two lanes of the same 16-lane group whose entries fall in
// the same quad (column mod 16 here) serialise.  The sum over a neuron's
// connections does not depend on their order, so each group of 16 neighbouring
// neurons gets its connections re-ordered such that in every step the 16 lanes
// touch 16 different quads whenever possible.  This plays the role the transposed
// sliced-ELL of Section III-A-3 plays for coalescing weight reads: a layout
// decision made once, before inference.
//
// How.  32 rounds, one per step.  In each round a maximum bipartite matching
// lanes <-> quads is built (augmenting paths), quads being offered in priority
// order: first those whose remaining connections equal or exceed the remaining
// steps (they must be served now or cost an extra cycle later), then by remaining
// count.  A lane left unmatched takes a connection from the quad that is least
// loaded in this round.  Cost = sum over rounds of the largest quad
// multiplicity; the lower bound is max(32, busiest quad's total).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define SPDNN_HD __host__ __device__
#else
#define SPDNN_HD
#endif

namespace spdnn {

constexpr int kGroup = 16;  // lanes served per clock by a 16-byte LDS read = quads per 256-byte bank row

// Working memory of one group (1104 bytes).  On the device it lives in LDS.
struct OrderScratch {
    uint8_t cnt[kGroup][16];   // connections of lane l still unplaced, per quad
    uint8_t end[kGroup][16];   // end of quad q's bucket in sorted[l]
    uint8_t sorted[kGroup][32];  // lane l's connection numbers, bucketed by quad
    uint16_t adj[16];          // adj[q]: lanes that still have a connection in quad q
    uint16_t remq[16];         // connections still unplaced in quad q over the whole group
    uint8_t reml[kGroup];      // connections of lane l still unplaced
};

SPDNN_HD inline unsigned nib_get(uint64_t w, int i) { return (unsigned)(w >> (4 * i)) & 15u; }
SPDNN_HD inline uint64_t nib_set(uint64_t w, int i, unsigned v) {
    return (w & ~(15ull << (4 * i))) | ((uint64_t)(v & 15u) << (4 * i));
}
SPDNN_HD inline int ctz16(unsigned m) {
    int n = 0;
    while (!(m & 1u)) {
        m >>= 1;
        ++n;
    }
    return n;
}

// quad_of(l, k), k < 32: quad (0..15) of connection k of lane l, or 255 if there is no
// such connection (a lane may have fewer than 32, or none).  emit(l, step, k):
// connection k of lane l is placed at step `step` < nsteps.  nsteps must be at least
// the largest number of connections any lane has; every existing connection is emitted
// exactly once, at most one per lane and step; a lane with fewer connections than
// steps sits out the steps in which it would collide.
template <typename QuadOf, typename Emit>
SPDNN_HD inline void order_group(OrderScratch& S, int nsteps, QuadOf quad_of, Emit emit) {
    uint16_t* adj = S.adj;
    uint16_t* remq = S.remq;
    for (int q = 0; q < 16; ++q) {
        adj[q] = 0;
        remq[q] = 0;
    }
    unsigned live = 0;  // lanes that have connections at all
    for (int l = 0; l < kGroup; ++l) {
        for (int q = 0; q < 16; ++q) S.cnt[l][q] = 0;
        for (int k = 0; k < 32; ++k) {
            const unsigned q = quad_of(l, k);
            if (q < 16) S.cnt[l][q]++;
        }
        unsigned run = 0;
        for (int q = 0; q < 16; ++q) {
            run += S.cnt[l][q];
            S.end[l][q] = (uint8_t)run;
            if (S.cnt[l][q]) adj[q] |= (uint16_t)(1u << l);
            remq[q] += S.cnt[l][q];
        }
        if (run) live |= 1u << l;
        S.reml[l] = (uint8_t)run;
        // counting sort of the connection numbers by quad (stable)
        uint8_t fill[16];
        for (int q = 0; q < 16; ++q) fill[q] = (uint8_t)(S.end[l][q] - S.cnt[l][q]);
        for (int k = 0; k < 32; ++k) {
            const unsigned q = quad_of(l, k);
            if (q < 16) S.sorted[l][fill[q]++] = (uint8_t)k;
        }
    }
    for (int step = 0; step < nsteps; ++step) {
        const int left = nsteps - step;
        uint64_t lane_of = 0, quad_of_l = 0, par = 0;  // nibble arrays
        unsigned mq = 0, ml = 0;                        // matched quads / lanes
        unsigned done = 0;                              // quads already offered
        for (int r = 0; r < 16; ++r) {
            // next quad by priority
            int q0 = -1;
            int best = -1;
            for (int q = 0; q < 16; ++q) {
                if ((done >> q) & 1u) continue;
                const int key = (remq[q] >= left ? 4096 : 0) + remq[q];
                if (key > best) {
                    best = key;
                    q0 = q;
                }
            }
            done |= 1u << q0;
            if (remq[q0] == 0) break;  // the rest are empty too
            // breadth-first search for an augmenting path from q0 to a free lane
            uint64_t queue = (uint64_t)q0;
            int head = 0, tail = 1;
            unsigned seen = 0;
            int found = -1;
            while (head < tail && found < 0) {
                const int q = (int)nib_get(queue, head++);
                unsigned cand = adj[q] & ~seen;
                while (cand) {
                    const int l = ctz16(cand);
                    cand &= cand - 1;
                    seen |= 1u << l;
                    par = nib_set(par, l, (unsigned)q);
                    if (!((ml >> l) & 1u)) {
                        found = l;
                        break;
                    }
                    queue = nib_set(queue, tail++, nib_get(quad_of_l, l));
                }
            }
            if (found < 0) continue;
            int cur = found;
            for (;;) {
                const int q = (int)nib_get(par, cur);
                const int next = (int)nib_get(lane_of, q);  // meaningful only if q was matched
                lane_of = nib_set(lane_of, q, (unsigned)cur);
                quad_of_l = nib_set(quad_of_l, cur, (unsigned)q);
                ml |= 1u << cur;
                const bool first = (q == q0);
                mq |= 1u << q;
                if (first) break;
                cur = next;
            }
        }
        // lanes without a quad of their own share the least loaded one they can use
        uint64_t mult = 0;  // nibble: uses of quad q in this step (saturates at 15)
        for (int l = 0; l < kGroup; ++l)
            if ((ml >> l) & 1u) {
                const int q = (int)nib_get(quad_of_l, l);
                mult = nib_set(mult, q, nib_get(mult, q) + 1);
            }
        unsigned placed = ml;  // lanes that place a connection in this step
        for (int l = 0; l < kGroup; ++l) {
            if (!((live >> l) & 1u) || ((ml >> l) & 1u)) continue;
            if ((int)S.reml[l] < left) continue;  // has slack: sits this step out
            int bq = -1;
            int bkey = 1 << 30;
            for (int q = 0; q < 16; ++q) {
                if (!S.cnt[l][q]) continue;
                const int key = (int)nib_get(mult, q) * 65536 - ((int)remq[q] - left) * 64 - (int)S.cnt[l][q];
                if (key < bkey) {
                    bkey = key;
                    bq = q;
                }
            }
            quad_of_l = nib_set(quad_of_l, l, (unsigned)bq);
            placed |= 1u << l;
            const unsigned m = nib_get(mult, bq);
            mult = nib_set(mult, bq, m < 15 ? m + 1 : 15);
        }
        // place the chosen connections
        for (int l = 0; l < kGroup; ++l) {
            if (!((placed >> l) & 1u)) continue;
            const int q = (int)nib_get(quad_of_l, l);
            const int k = S.sorted[l][S.end[l][q] - S.cnt[l][q]];
            S.cnt[l][q]--;
            remq[q]--;
            if (!S.cnt[l][q]) adj[q] &= (uint16_t)~(1u << l);
            if (--S.reml[l] == 0) live &= ~(1u << l);
            emit(l, step, k);
        }
    }
}

// Cost model used by tests: LDS cycles of one group's 32 steps (largest quad
// multiplicity per step, summed).  quad_at(l, step) as placed.
template <typename QuadAt>
SPDNN_HD inline int order_cost(QuadAt quad_at) {
    int total = 0;
    for (int step = 0; step < 32; ++step) {
        int m[16] = {0};
        int mx = 0;
        for (int l = 0; l < kGroup; ++l) {
            const unsigned q = quad_at(l, step);
            if (q < 16 && ++m[q] > mx) mx = m[q];
        }
        total += mx;
    }
    return total;
}

// The same ordering problem for the kernel that reads two rows per LDS entry (ds_read_b64):
// gfx950 serves such a read half a wave at a time -- lanes 0..31, then 32..63 -- from 32 "pairs"
// of neighbouring 4-byte banks (measured with a pairwise-conflict probe), so a group is 32
// neighbouring neurons and a step is conflict-free when their 32 entries fall in 32 different
// bank pairs.  Every lane has exactly 32 connections and places one per step.
//
// Per step: a maximum bipartite matching pairs <-> lanes by augmenting paths (breadth-first),
// pairs offered by urgency -- first those that hold at least as many unplaced connections as
// there are steps left (they must be served in every remaining step or cost an extra cycle
// later), then by what they still hold.  A lane left without a pair of its own shares the least
// used pair it can.  Cost of a group = sum over the steps of the largest pair multiplicity;
// the lower bound is max(32, the busiest pair's total).
constexpr int kGroup32 = 32;
struct Order32Scratch {
    uint8_t pair[kGroup32][32];   // bank pair of connection k of lane l
    uint32_t unplaced[kGroup32];  // connections of lane l not placed yet (bit k)
    uint32_t adj[32];             // lanes that still have a connection in pair q
    uint16_t remq[32];            // connections not placed yet in pair q, whole group
    int8_t lane_of_pair[32];      // matching of the current step
    int8_t pair_of_lane[kGroup32];
    int8_t parent[kGroup32];      // pair from which the search reached lane l
    uint8_t queue[36];
    uint8_t mult[32];             // lanes using pair q in the current step
};

SPDNN_HD inline int ctz32(uint32_t m) {
    int n = 0;
    while (!(m & 1u)) {
        m >>= 1;
        ++n;
    }
    return n;
}

// pair_of(l, k): bank pair (0..31) of connection k of lane l.  emit(l, step, k): connection k of
// lane l goes to step `step`; called exactly once per (l, k), once per (l, step).
template <typename PairOf, typename Emit>
SPDNN_HD inline void order_group32(Order32Scratch& S, PairOf pair_of, Emit emit) {
    for (int l = 0; l < kGroup32; ++l) {
        for (int k = 0; k < 32; ++k) S.pair[l][k] = (uint8_t)(pair_of(l, k) & 31u);
        S.unplaced[l] = 0xFFFFFFFFu;
    }
    for (int step = 0; step < 32; ++step) {
        const int left = 32 - step;
        for (int q = 0; q < 32; ++q) {
            S.adj[q] = 0;
            S.remq[q] = 0;
            S.lane_of_pair[q] = -1;
            S.mult[q] = 0;
        }
        for (int l = 0; l < kGroup32; ++l) {
            S.pair_of_lane[l] = -1;
            uint32_t m = S.unplaced[l];
            while (m) {
                const int k = ctz32(m);
                m &= m - 1;
                const int q = S.pair[l][k];
                S.adj[q] |= 1u << l;
                S.remq[q]++;
            }
        }
        uint32_t done = 0;  // pairs already offered
        for (int r = 0; r < 32; ++r) {
            int q0 = -1, best = -1;
            for (int q = 0; q < 32; ++q) {
                if ((done >> q) & 1u) continue;
                const int key = (S.remq[q] >= left ? 4096 : 0) + S.remq[q];
                if (key > best) {
                    best = key;
                    q0 = q;
                }
            }
            done |= 1u << q0;
            if (S.remq[q0] == 0) break;  // the rest are empty too
            // breadth-first search for an augmenting path from pair q0 to a lane without a pair
            int head = 0, tail = 0, found = -1;
            uint32_t seen = 0;
            S.queue[tail++] = (uint8_t)q0;
            while (head < tail && found < 0) {
                const int q = S.queue[head++];
                uint32_t cand = S.adj[q] & ~seen;
                while (cand) {
                    const int l = ctz32(cand);
                    cand &= cand - 1;
                    seen |= 1u << l;
                    S.parent[l] = (int8_t)q;
                    if (S.pair_of_lane[l] < 0) {
                        found = l;
                        break;
                    }
                    S.queue[tail++] = (uint8_t)S.pair_of_lane[l];  // a lane is seen once: at most 32 entries follow q0
                }
            }
            if (found < 0) continue;
            for (int cur = found;;) {
                const int q = S.parent[cur];
                const int next = S.lane_of_pair[q];  // the lane that gives q up (meaningful unless q == q0)
                S.lane_of_pair[q] = (int8_t)cur;
                S.pair_of_lane[cur] = (int8_t)q;
                if (q == q0) break;
                cur = next;
            }
        }
        for (int l = 0; l < kGroup32; ++l)
            if (S.pair_of_lane[l] >= 0) S.mult[S.pair_of_lane[l]]++;
        for (int l = 0; l < kGroup32; ++l) {
            if (S.pair_of_lane[l] >= 0) continue;
            int bq = -1, bkey = 1 << 30;
            for (int q = 0; q < 32; ++q) {
                if (!((S.adj[q] >> l) & 1u)) continue;
                const int key = (int)S.mult[q] * 65536 - (int)S.remq[q];
                if (key < bkey) {
                    bkey = key;
                    bq = q;
                }
            }
            S.pair_of_lane[l] = (int8_t)bq;
            S.mult[bq]++;
        }
        for (int l = 0; l < kGroup32; ++l) {
            const int q = S.pair_of_lane[l];
            uint32_t m = S.unplaced[l];
            int k = -1;
            while (m) {
                const int kk = ctz32(m);
                m &= m - 1;
                if (S.pair[l][kk] == q) {
                    k = kk;
                    break;
                }
            }
            S.unplaced[l] &= ~(1u << k);
            emit(l, step, k);
        }
    }
}

}  // namespace spdnn
